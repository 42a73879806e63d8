// dQ on bf16 MFMA, variant that shares the coarse levels (B = 16, 32 or 64, d = 64 or 128, N a multiple of 256,
// at most 64 level-0 tiles per list); see attn_fwd_shared.hip for the decomposition (a workgroup of 8 waves owns
// 128 consecutive queries, which use the same lists at every level >= 1, every wave one 16-query tile; the coarse
// key/value tiles are staged once per workgroup in LDS, the level-0 tiles are walked per query tile).
// Per tile and query block:  S^T = K Q^T, dP^T = V dO^T  ->  dS^T = P^T o (dP^T - D)  ->  dQ^T += K^T dS^T,
// with K read from LDS both row-wise (first product) and transposed (last product).
// The kernel also produces D = rowsum(dO o O) for its queries and stores it for the key-major kernels.
#include <type_traits>

#include "mfma_common.h"

namespace llsa {

typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr_t;
__device__ __forceinline__ u32x4 gload16b(const char *base, unsigned off) {
    return *reinterpret_cast<gvec_ptr_t>(reinterpret_cast<const __attribute__((address_space(1))) char *>(
        reinterpret_cast<uintptr_t>(base)) + off);
}
__device__ __forceinline__ bf16x8 to_bf16x8(u32x4 v) {
    union { u32x4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}
__device__ __forceinline__ float bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// NB = fine query blocks per wave (1 or 2); a workgroup owns 8 * NB consecutive blocks, all siblings
template <int D, int NB>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(D == 64 ? 4 : 2)))
dq_shared_kernel(LevelTable t, const uint16_t *__restrict__ Q, const uint16_t *__restrict__ O,
                 const uint16_t *__restrict__ dO, const float *__restrict__ LSE, float *__restrict__ Dsum,
                 uint16_t *__restrict__ dQ, int64_t N, int64_t total_wgs) {
    constexpr int KS = D / 32, NT = D / 16, STRIDE = D * 2 + 32, PARTS = D / 8, TILE = 32 * STRIDE;
    constexpr int RND = (2 * 32 * PARTS) / 512, VCH = D / 16, KPU = 64 / PARTS;
    // Phase B: per wave a K tile (row-wise and transposed reads) and a V tile (row-wise reads only; 16 bytes of
    // padding keep it smaller).  Phase A's two double-buffered [K | V] tiles live in the first 4 TILE bytes of the
    // same memory; a workgroup barrier separates the phases.
    constexpr int VSTRIDE = D * 2 + 16, VTILE = 32 * VSTRIDE;
    __shared__ __attribute__((aligned(16))) char lds[8 * (TILE + VTILE)];
    static_assert(4 * TILE <= 8 * (TILE + VTILE), "phase A's buffers must fit");
    auto sh = [&](int buf, int which) { return lds + (buf * 2 + which) * TILE; };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t groups = N / (128 * NB);                            // workgroups per head (8 * NB query blocks each)
    const int64_t wg = xcd_contiguous(blockIdx.x, total_wgs);
    const int64_t bh = wg / groups, blk0 = (wg % groups) * (8 * NB);
    const float sc2 = t.scale * kLog2e;

    bf16x8 qop[NB][KS], gop[NB][KS];
    f32x4 acc[NB][NT];
    float lse2[NB], delta[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int64_t qrow = bh * N + (blk0 + NB * wave + b) * 16 + i16;
        float dl = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            qop[b][s] = ld_bf16x8(Q + qrow * D + g * 8 + 32 * s);
            const u32x4 gw = *reinterpret_cast<const u32x4 *>(dO + qrow * D + g * 8 + 32 * s);
            const u32x4 ow = *reinterpret_cast<const u32x4 *>(O + qrow * D + g * 8 + 32 * s);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dl = fmaf(bf_lo(gw[e]), bf_lo(ow[e]), dl);
                dl = fmaf(bf_hi(gw[e]), bf_hi(ow[e]), dl);
            }
            gop[b][s] = to_bf16x8(gw);
        }
        delta[b] = rows_sum(dl);
        if (g == 0) Dsum[qrow] = delta[b];
        lse2[b] = LSE[qrow] * kLog2e;
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[b][n] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // dS^T of query block b for one tile and dQ^T += K^T dS^T with the K tile at `kt`
    auto ds_dq = [&](auto bsel, f32x4 s0, f32x4 s1, f32x4 dp0, f32x4 dp1, int c0, int c1, float b0, float b1,
                     const char *kt) {
        constexpr int b = decltype(bsel)::value;
        f32x4 s[2] = {s0, s1};
        const f32x4 dp[2] = {dp0, dp1};
        const float c2[2] = {b0 - lse2[b], b1 - lse2[b]};
        const int c[2] = {c0, c1};
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[h][r], sc2, c2[h]));
                s[h][r] = p * (dp[h][r] - delta[b]);
            }
        if (c[0] < 16 || c[1] < 16) {                                 // ragged or absent block contributes nothing
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (4 * g + r >= c[h]) s[h][r] = 0.f;
        }
        const bf16x8 dsop = pack8(s[0], s[1]);
        const char *base = kt + (4 * g + (i16 >> 2)) * STRIDE + (i16 & 3) * 8;
#pragma unroll
        for (int n = 0; n < NT; ++n)
            acc[b][n] = mfma16(lds_tr_pair(base + n * 32, base + 16 * STRIDE + n * 32), dsop, acc[b][n]);
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;

    // The level-0 lists of this wave's NB query blocks, fetched now so that phase B does not wait for them:
    // lane (64 / NB) b + j holds the first token of 16-token tile j of query tile b's list (as in the forward kernel).
    const int nb0 = t.bseg[1];
    int tok0 = 0;
    {
        const int b = lane / (64 / NB), j = lane % (64 / NB);
        if (j < nb0) {
            const int64_t row = (blk0 + NB * wave + b) >> t.ls;
            tok0 = (t.I[0][(bh * t.rows[0] + row) * t.Kl[0] + (j >> t.ls)] << t.lb) + ((j & ((1 << t.ls) - 1)) << 4);
        }
    }

    // ------------------------------------------------------------------ phase A: shared coarse levels
    const int c_begin = t.nlev > 1 ? t.bseg[1] : t.bseg[t.nlev];
    const int nbc = t.bseg[t.nlev] - c_begin;
    if (nbc > 0) {
        BlockTable ctab;
        ctab.fill_once(t, bh, blk0, c_begin, lane, wave, D, reinterpret_cast<uint32_t *>(lds + 4 * TILE));
        // Staging round r of this wave: 64 consecutive 16-byte chunks of the [K | V] tile, i.e. 64 / PARTS key rows of
        // one half of K or of V, the same choice for the whole wave (d = 64: one round, waves 0-3 stage K, waves 4-7
        // V; d = 128: round 0 stages K, round 1 V).
        u32x4 sreg[RND];
        int s_half[RND];
        unsigned s_off[RND];
#pragma unroll
        for (int r = 0; r < RND; ++r) {
            const int key0 = ((64 * wave + 512 * r) % (32 * PARTS)) / PARTS;   // the wave's first key row in round r
            s_half[r] = key0 >> 4;
            s_off[r] = (unsigned)((((key0 & 15) + lane / PARTS) * D + (lane % PARTS) * 8) * 2);
        }
        const bool v_wave = RND == 1 && wave >= 4;
        uint64_t sptr = v_wave ? ctab.vptr : ctab.kptr;               // d = 64: the tensor this wave stages
        auto load_shared = [&](int u) {
            if (u > 0 && ((2 * u) & 63) == 0) {
                ctab.fill(t, bh, blk0, c_begin, (2 * u) >> 6, lane, D);
                sptr = v_wave ? ctab.vptr : ctab.kptr;
            }
#pragma unroll
            for (int r = 0; r < RND; ++r) {
                const bool have = 2 * u + s_half[r] < nbc;
                const int j = (have ? 2 * u + s_half[r] : 2 * u) & 63;
                const int cnt = have ? ctab.count(j) : 0;
                const char *src = RND == 1 ? BlockTable::rl_ptr(sptr, j) : (r == 0 ? ctab.K(j) : ctab.V(j));
                unsigned off = s_off[r];
                if (cnt < 16) {                                       // ragged or absent block: re-read its last valid row
                    const int row = min((int)(off / (D * 2)), max(cnt, 1) - 1);
                    off = (unsigned)(row * D * 2) + off % (D * 2);
                }
                sreg[r] = gload16b(src, off);
            }
        };
        auto store_shared = [&](int buf) {
#pragma unroll
            for (int r = 0; r < RND; ++r) {
                const int cc = tid + 512 * r, which = cc / (32 * PARTS), c = cc % (32 * PARTS);
                *reinterpret_cast<u32x4 *>(sh(buf, which) + (c / PARTS) * STRIDE + (c % PARTS) * 16) = sreg[r];
            }
        };
        const int ntile = (nbc + 1) >> 1;
        load_shared(0);
        for (int u = 0; u < ntile; ++u) {
            const int buf = u & 1;
            store_shared(buf);
            int cnt[2];
            float bias2[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const bool have = 2 * u + h < nbc;
                const int j = have ? 2 * u + h : 2 * u;
                cnt[h] = have ? ctab.count(j & 63) : 0;
                bias2[h] = ctab.bias(j & 63);
            }
            __syncthreads();
            if (u + 1 < ntile) load_shared(u + 1);
            const char *kt = sh(buf, 0), *vt = sh(buf, 1);
            // one query block at a time keeps the live score registers low (the row-wise operands are
            // re-read from LDS for the second block)
            auto scores = [&](auto bsel) {
                constexpr int b = decltype(bsel)::value;
                f32x4 s[2], dp[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
                    dp[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        const int off = (h * 16 + i16) * STRIDE + g * 16 + ks * 64;
                        s[h] = mfma16(*reinterpret_cast<const bf16x8 *>(kt + off), qop[b][ks], s[h]);
                        dp[h] = mfma16(*reinterpret_cast<const bf16x8 *>(vt + off), gop[b][ks], dp[h]);
                    }
                }
                ds_dq(bsel, s[0], s[1], dp[0], dp[1], cnt[0], cnt[1], bias2[0], bias2[1], kt);
            };
            scores(B0{});
            if constexpr (NB > 1) scores(B1{});
        }
    }

    // ------------------------------------------------------------------ phase B: own level-0 blocks
    // K and V rows are fetched with 8 consecutive lanes per 128-byte row (whole cache lines per instruction: loading
    // the MFMA operand layout straight from memory, 16 rows x half a line per instruction, caps the gather rate at a
    // third of what the L2 delivers) and reach the operand layouts through the wave's own LDS tiles.
    __syncthreads();                                                  // phase A's buffers are free
    char *my = lds + wave * (TILE + VTILE), *my_v = my + TILE;
    const char *K0 = static_cast<const char *>(t.K[0]), *V0 = static_cast<const char *>(t.V[0]);
    unsigned voff[VCH];
#pragma unroll
    for (int u = 0; u < VCH; ++u) voff[u] = (unsigned)((((lane / PARTS + KPU * u) & 15) * D + (lane % PARTS) * 8) * 2);

    auto phase_b = [&](auto bsel) {
        constexpr int b = decltype(bsel)::value;
        u32x4 kreg[VCH], vreg[VCH];
        auto load_tile = [&](int j0) {
            int64_t off[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int j = (j0 + h < nb0) ? j0 + h : j0;           // an absent second half re-reads the first
                off[h] = (bh * N + __builtin_amdgcn_readlane(tok0, (64 / NB) * b + j)) * (D * 2);
            }
#pragma unroll
            for (int u = 0; u < VCH; ++u) {
                kreg[u] = gload16b(K0 + off[(KPU * u) >> 4], voff[u]);
                vreg[u] = gload16b(V0 + off[(KPU * u) >> 4], voff[u]);
            }
        };
        load_tile(0);
        for (int j0 = 0; j0 < nb0; j0 += 2) {
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int u = 0; u < VCH; ++u) {
                *reinterpret_cast<u32x4 *>(my + (lane / PARTS + KPU * u) * STRIDE + (lane % PARTS) * 16) = kreg[u];
                *reinterpret_cast<u32x4 *>(my_v + (lane / PARTS + KPU * u) * VSTRIDE + (lane % PARTS) * 16) = vreg[u];
            }
            __builtin_amdgcn_wave_barrier();
            if (j0 + 2 < nb0) load_tile(j0 + 2);                      // the registers are free again
            f32x4 s[2], dp[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
                dp[h] = f32x4{0.f, 0.f, 0.f, 0.f};
                const char *krow = my + (h * 16 + i16) * STRIDE + g * 16, *vrow = my_v + (h * 16 + i16) * VSTRIDE + g * 16;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    s[h] = mfma16(*reinterpret_cast<const bf16x8 *>(krow + ks * 64), qop[b][ks], s[h]);
                    dp[h] = mfma16(*reinterpret_cast<const bf16x8 *>(vrow + ks * 64), gop[b][ks], dp[h]);
                }
            }
            const int c1 = (j0 + 1 < nb0) ? 16 : 0;
            ds_dq(bsel, s[0], s[1], dp[0], dp[1], 16, c1, 0.f, 0.f, my);
        }
    };
    phase_b(B0{});
    if constexpr (NB > 1) phase_b(B1{});

#pragma unroll
    for (int b = 0; b < NB; ++b) {
        uint16_t *orow = dQ + (bh * N + (blk0 + NB * wave + b) * 16 + i16) * D + 4 * g;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            u32x2 w;
            w[0] = pack_bf16(acc[b][n][0] * t.scale, acc[b][n][1] * t.scale);
            w[1] = pack_bf16(acc[b][n][2] * t.scale, acc[b][n][3] * t.scale);
            *reinterpret_cast<u32x2 *>(orow + n * 16) = w;
        }
    }
}

hipError_t launch_dq_shared(const Plan &p, const LevelTable &t, const void *Q, const void *O, const void *dO,
                            const float *LSE, float *D, void *dQ, hipStream_t s) {
    const int64_t wgs = (int64_t)p.bh * (p.N / 128);                  // one query block per wave: 8 per workgroup
    if (p.d == 128) {
        dq_shared_kernel<128, 1><<<dim3((unsigned)wgs), 512, 0, s>>>(t, (const uint16_t *)Q, (const uint16_t *)O,
                                                                      (const uint16_t *)dO, LSE, D, (uint16_t *)dQ, p.N, wgs);
        return hipGetLastError();
    }
    dq_shared_kernel<64, 1><<<dim3((unsigned)wgs), 512, 0, s>>>(t, (const uint16_t *)Q, (const uint16_t *)O,
                                                             (const uint16_t *)dO, LSE, D, (uint16_t *)dQ, p.N, wgs);
    return hipGetLastError();
}

}  // namespace llsa
