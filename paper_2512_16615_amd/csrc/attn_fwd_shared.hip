// Attention forward over the gathered lists on bf16 MFMA, variant that shares the coarse levels
// (B = 16, 32 or 64, d = 64 or 128, N a multiple of 256, at most 64 level-0 tiles of 16 tokens per list).
//
// 256 consecutive queries (B = 16: the 16 fine query blocks under one level-1 query block) use the same lists at
// every level >= 1 (Alg. 1, enrichment loop: block i reads row i / B^l of I^(l)), i.e. the same coarse key/value
// tokens.  One workgroup of 4 or 8 waves owns such a group or half of one; every wave owns one or two of its
// 16-query tiles.
//   Phase A (levels >= 1): the workgroup stages each tile of two 16-token blocks (K and V rows) once in
//     LDS, double-buffered; every wave reads the K operand once and multiplies it with both of its query
//     blocks, likewise the transposed V operand, so the gather traffic of the coarse tokens is paid once
//     per 128 or 256 queries instead of once per 16.
//   Phase B (level 0): each wave walks the level-0 tiles of each of its query tiles' lists; their K and V rows are
//     fetched as whole cache lines and reach the operand layouts through the wave's private LDS tiles.
// Score tiles are computed transposed (S^T = K Q^T) so that the accumulator layout (4 keys x 1 query per
// lane) is the B operand of O^T += V^T P^T; see mfma_common.h for the register layouts.
#include <type_traits>

#include "mfma_common.h"

namespace llsa {

typedef const __attribute__((address_space(1))) u32x4 *gvec_ptr;
__device__ __forceinline__ u32x4 gload16(const char *base, unsigned off) {
    return *reinterpret_cast<gvec_ptr>(reinterpret_cast<const __attribute__((address_space(1))) char *>(
        reinterpret_cast<uintptr_t>(base)) + off);
}
constexpr float kLazy = 12.f;       // a query's softmax reference is raised only when a logit exceeds it by 2^kLazy

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) {
    union { u32x4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

// NB = fine query blocks per wave (1 or 2), NW = waves per workgroup (4 or 8); a workgroup owns NW * NB consecutive
// blocks, all siblings
template <int D, int NB, int NW = 8>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(D == 64 ? 4 : 2))) attn_fwd_shared_kernel(LevelTable t, const uint16_t *__restrict__ Q,
                                                               uint16_t *__restrict__ O, float *__restrict__ LSE,
                                                               int64_t N, int64_t total_wgs) {
    constexpr int KS = D / 32, NT = D / 16, STRIDE = D * 2 + 32, PARTS = D / 8, TILE = 32 * STRIDE;
    constexpr int NTHR = 64 * NW;
    constexpr int RND = (2 * 32 * PARTS) / NTHR;        // staging rounds of the workgroup per shared tile (K and V)
    static_assert(RND == 1 || NTHR == 32 * PARTS, "with two rounds, round 0 is the K half and round 1 the V half");
    constexpr int VCH = D / 16, KPU = 64 / PARTS;       // private V staging of one wave (phase B)
    // Phase B: per wave a K tile (row-wise reads: rows 32 bytes apart in the banks) and a V tile (transposed reads only:
    // 16 bytes of padding do).  Phase A's two double-buffered [K | V] tiles live in the first 4 TILE bytes of the same
    // memory; a workgroup barrier separates the phases.
    constexpr int VSTRIDE = D * 2 + 16, VTILE = 32 * VSTRIDE;
    __shared__ __attribute__((aligned(16))) char lds[NW * (TILE + VTILE)];
    static_assert(4 * TILE + 6 * 64 * 4 <= NW * (TILE + VTILE), "phase A's buffers and the block table must fit");
    auto sh = [&](int buf, int which) { return lds + (buf * 2 + which) * TILE; };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t groups = N / (16 * NW * NB);                        // workgroups per head
    const int64_t wg = xcd_contiguous(blockIdx.x, total_wgs);
    const int64_t bh = wg / groups, blk0 = (wg % groups) * (NW * NB);
    const float sc2 = t.scale * kLog2e;

    bf16x8 qop[NB][KS];
    f32x4 acc[NB][NT];
    float m[NB], mthr[NB], lsum[NB];                                  // reference, reference + kLazy, this lane's row-sum share
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const uint16_t *qrow = Q + (bh * N + (blk0 + NB * wave + b) * 16 + i16) * D + g * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) qop[b][s] = ld_bf16x8(qrow + 32 * s);
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[b][n] = f32x4{0.f, 0.f, 0.f, 0.f};
        m[b] = mthr[b] = -INFINITY;
        lsum[b] = 0.f;
    }

    // softmax update of query block b for one tile (s0 / s1: raw S^T of the two halves) and O^T += V^T P^T
    // with the V tile at `vt` (row-major, VS bytes per key row).  The running reference m[b] of a query is not its
    // exact maximum: it is raised (and the accumulators rescaled) only when a logit exceeds it by more than kLazy
    // (log2 units), so probabilities stay below 2^kLazy, which costs fp32 / bf16 no precision, and a tile's usual
    // cost is a lane-local maximum and one compare.  Scale, level weight and reference are folded into the one
    // multiply-add in front of the exponential.
    auto softmax_pv = [&](auto bsel, f32x4 s0, f32x4 s1, int c0, int c1, float b0, float b1, const char *vt, auto vstride,
                          auto joint) -> bf16x8 {
        constexpr int b = decltype(bsel)::value;
        constexpr int VS = decltype(vstride)::value;                  // bytes between the V tile's key rows
        f32x4 s[2] = {s0, s1};
        if (c0 < 16 || c1 < 16) {                                     // ragged or absent block: mask
            const int c[2] = {c0, c1};
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (4 * g + r >= c[h]) s[h][r] = -INFINITY;
        }
        const float mx0 = fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3]));
        const float mx1 = fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3]));
        const float z = fmaxf(fmaf(mx0, sc2, b0), fmaf(mx1, sc2, b1));       // this lane's largest logit (log2 units)
        if (__builtin_amdgcn_ballot_w64(z > mthr[b]) != 0) {          // some row outgrew its reference: rescale
            const float m_new = fmaxf(m[b], rows_max(z));
            const float alpha = __builtin_amdgcn_exp2f(m[b] - m_new);
            lsum[b] *= alpha;
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[b][n][r] *= alpha;
            m[b] = m_new;
            mthr[b] = m_new + kLazy;
        }
        const float cb[2] = {b0 - m[b], b1 - m[b]};
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s[h][r] = __builtin_amdgcn_exp2f(fmaf(s[h][r], sc2, cb[h]));
                lsum[b] += s[h][r];
            }
        const bf16x8 pop = pack8(s[0], s[1]);
        if constexpr (decltype(joint)::value) {
            return pop;                                               // the caller multiplies both blocks' P with one read of V
        } else {
            const char *base = vt + (4 * g + (i16 >> 2)) * VS + (i16 & 3) * 8;
#pragma unroll
            for (int n = 0; n < NT; ++n)
                acc[b][n] = mfma16(lds_tr_pair(base + n * 32, base + 16 * VS + n * 32), pop, acc[b][n]);
            return pop;
        }
    };
    using StrideA = std::integral_constant<int, STRIDE>;
    using StrideB = std::integral_constant<int, VSTRIDE>;
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;

    // The level-0 lists of this wave's NB query blocks, fetched now so that phase B does not wait for them:
    // lane (64 / NB) b + j holds the first token of 16-token tile j of query tile b's list (at most 64 / NB tiles;
    // a listed block of B tokens is B / 16 consecutive tiles, and B / 16 consecutive query tiles share a row of I^(0)).
    const int nb0 = t.bseg[1];                                        // level-0 tiles (the list always holds level 0)
    int tok0 = 0;
    {
        const int b = lane / (64 / NB), j = lane % (64 / NB);
        if (j < nb0) {
            const int64_t row = (blk0 + NB * wave + b) >> t.ls;
            tok0 = (t.I[0][(bh * t.rows[0] + row) * t.Kl[0] + (j >> t.ls)] << t.lb) + ((j & ((1 << t.ls) - 1)) << 4);
        }
    }

    // ------------------------------------------------------------------ phase A: shared coarse levels
    const int c_begin = t.nlev > 1 ? t.bseg[1] : t.bseg[t.nlev];     // first coarse block of the list
    const int nbc = t.bseg[t.nlev] - c_begin;                         // coarse blocks
    if (nbc > 0) {
        BlockTable ctab;                                              // lane j: coarse block 64 * chunk + j
        ctab.fill_once(t, bh, blk0, c_begin, lane, wave, D, reinterpret_cast<uint32_t *>(lds + 4 * TILE));
        // Staging round r of this wave: 64 consecutive 16-byte chunks of the [K | V] tile, i.e. 64 / PARTS key rows of
        // one half of K or of V, the same choice for the whole wave.
        // (d = 64: one round, waves 0-3 stage K, waves 4-7 V; d = 128: round 0 stages K, round 1 V.)
        u32x4 sreg[RND];
        int s_half[RND];
        unsigned s_off[RND];
#pragma unroll
        for (int r = 0; r < RND; ++r) {
            const int key0 = ((64 * wave + NTHR * r) % (32 * PARTS)) / PARTS;   // the wave's first key row in round r
            s_half[r] = key0 >> 4;
            s_off[r] = (unsigned)((((key0 & 15) + lane / PARTS) * D + (lane % PARTS) * 8) * 2);
        }
        const bool v_wave = RND == 1 && wave >= 4;
        uint64_t sptr = v_wave ? ctab.vptr : ctab.kptr;               // d = 64: the tensor this wave stages
        auto load_shared = [&](int u) {                               // coarse blocks 2u, 2u + 1 -> registers
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
                sreg[r] = gload16(src, off);
            }
        };
        auto store_shared = [&](int buf) {
#pragma unroll
            for (int r = 0; r < RND; ++r) {
                const int cc = tid + NTHR * r, which = cc / (32 * PARTS), c = cc % (32 * PARTS);
                *reinterpret_cast<u32x4 *>(sh(buf, which) + (c / PARTS) * STRIDE + (c % PARTS) * 16) = sreg[r];
            }
        };
        const int ntile = (nbc + 1) >> 1;
        load_shared(0);
        for (int u = 0; u < ntile; ++u) {
            const int buf = u & 1;
            store_shared(buf);
            // per-half fields of this tile, before the table may be refilled for the next one
            int cnt[2];
            float bias2[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const bool have = 2 * u + h < nbc;
                const int j = have ? 2 * u + h : 2 * u;
                cnt[h] = have ? ctab.count(j & 63) : 0;
                bias2[h] = ctab.bias(j & 63);
            }
            __syncthreads();                                          // tile u visible; buffer buf^1 free again
            if (u + 1 < ntile) load_shared(u + 1);
            const char *kt = sh(buf, 0), *vt = sh(buf, 1);
            bf16x8 kop[2][KS];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    kop[h][ks] = *reinterpret_cast<const bf16x8 *>(kt + (h * 16 + i16) * STRIDE + g * 16 + ks * 64);
            f32x4 s[NB][2];
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    s[b][h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) s[b][h] = mfma16(kop[h][ks], qop[b][ks], s[b][h]);
                }
            if constexpr (NB > 1) {                                   // both blocks' P first, then one transposing read of V for both
                const bf16x8 p0 = softmax_pv(B0{}, s[0][0], s[0][1], cnt[0], cnt[1], bias2[0], bias2[1], vt, StrideA{}, std::true_type{});
                const bf16x8 p1 = softmax_pv(B1{}, s[NB - 1][0], s[NB - 1][1], cnt[0], cnt[1], bias2[0], bias2[1], vt, StrideA{}, std::true_type{});
                const char *base = vt + (4 * g + (i16 >> 2)) * STRIDE + (i16 & 3) * 8;
#pragma unroll
                for (int n = 0; n < NT; ++n) {
                    const bf16x8 vtr = lds_tr_pair(base + n * 32, base + 16 * STRIDE + n * 32);
                    acc[0][n] = mfma16(vtr, p0, acc[0][n]);
                    acc[NB - 1][n] = mfma16(vtr, p1, acc[NB - 1][n]);
                }
            } else {
                softmax_pv(B0{}, s[0][0], s[0][1], cnt[0], cnt[1], bias2[0], bias2[1], vt, StrideA{}, std::false_type{});
            }
        }
    }

    // ------------------------------------------------------------------ phase B: own level-0 blocks
    // K and V rows are fetched with 8 consecutive lanes per 128-byte row (whole cache lines per instruction: loading
    // the MFMA operand layout straight from memory, 16 rows x half a line per instruction, caps the gather rate at a
    // third of what the L2 delivers) and reach the operand layouts through the wave's own LDS tiles.
    __syncthreads();                                                  // phase A's buffers are free
    char *my_k = lds + wave * (TILE + VTILE), *my_v = my_k + TILE;
    unsigned voff[VCH];
#pragma unroll
    for (int u = 0; u < VCH; ++u) voff[u] = (unsigned)((((lane / PARTS + KPU * u) & 15) * D + (lane % PARTS) * 8) * 2);

    // The tiles of the wave's NB query blocks form one stream: the next tile's rows are in flight during the
    // current tile's math, also across the border between the two blocks (tok0: fetched before phase A).
    u32x4 kreg[VCH], vreg[VCH];
    const char *K0 = static_cast<const char *>(t.K[0]), *V0 = static_cast<const char *>(t.V[0]);
    auto load_tile = [&](int b, int j0) {
        int64_t off[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int j = (j0 + h < nb0) ? j0 + h : j0;               // an absent second half re-reads the first
            off[h] = (bh * N + __builtin_amdgcn_readlane(tok0, (64 / NB) * b + j)) * (D * 2);
        }
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            kreg[u] = gload16(K0 + off[(KPU * u) >> 4], voff[u]);
            vreg[u] = gload16(V0 + off[(KPU * u) >> 4], voff[u]);
        }
    };
    auto phase_b = [&](auto bsel) {
        constexpr int b = decltype(bsel)::value;
        for (int j0 = 0; j0 < nb0; j0 += 2) {
            __builtin_amdgcn_wave_barrier();                          // one wave's LDS operations stay in order
#pragma unroll
            for (int u = 0; u < VCH; ++u) {
                *reinterpret_cast<u32x4 *>(my_k + (lane / PARTS + KPU * u) * STRIDE + (lane % PARTS) * 16) = kreg[u];
                *reinterpret_cast<u32x4 *>(my_v + (lane / PARTS + KPU * u) * VSTRIDE + (lane % PARTS) * 16) = vreg[u];
            }
            __builtin_amdgcn_wave_barrier();
            if (j0 + 2 < nb0) load_tile(b, j0 + 2);                   // the registers are free again: next tile's rows
            else if (b + 1 < NB) load_tile(b + 1, 0);                 // fly during all of this tile's math
            f32x4 s[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    s[h] = mfma16(*reinterpret_cast<const bf16x8 *>(my_k + (h * 16 + i16) * STRIDE + g * 16 + ks * 64), qop[b][ks], s[h]);
            }
            const int c1 = (j0 + 1 < nb0) ? 16 : 0;                   // level-0 blocks are always full
            softmax_pv(bsel, s[0], s[1], 16, c1, 0.f, 0.f, my_v, StrideB{}, std::false_type{});
        }
    };
    load_tile(0, 0);
    phase_b(B0{});
    if constexpr (NB > 1) phase_b(B1{});

    // ------------------------------------------------------------------ epilogue
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const float l = rows_sum(lsum[b]);
        const float inv = 1.f / l;
        const int64_t row = bh * N + (blk0 + NB * wave + b) * 16 + i16;
        uint16_t *orow = O + row * D + 4 * g;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            u32x2 w;
            w[0] = pack_bf16(acc[b][n][0] * inv, acc[b][n][1] * inv);
            w[1] = pack_bf16(acc[b][n][2] * inv, acc[b][n][3] * inv);
            *reinterpret_cast<u32x2 *>(orow + n * 16) = w;
        }
        if (g == 0) LSE[row] = (m[b] + __builtin_amdgcn_logf(l)) * kLn2;
    }
}

hipError_t launch_attn_fwd_shared(const Plan &p, const LevelTable &t, const void *Q, void *O, float *LSE,
                                  hipStream_t s) {
    if (p.d == 64 && (p.Kl[0] << (p.lb - 4)) <= 32) { // two query blocks per wave (measured faster than one)
        // workgroups of four waves (8 query blocks), four per CU: same occupancy as two of eight waves, cheaper barriers
        // (measured 225 against 229 us)
        const int64_t wgs = (int64_t)p.bh * (p.N / 128);
        attn_fwd_shared_kernel<64, 2, 4><<<dim3((unsigned)wgs), 256, 0, s>>>(t, (const uint16_t *)Q, (uint16_t *)O, LSE, p.N,
                                                                              wgs);
    } else if (p.d == 64) {                           // K_0 > 32: both level-0 lists would not fit one register
        const int64_t wgs = (int64_t)p.bh * (p.N / 128);
        attn_fwd_shared_kernel<64, 1><<<dim3((unsigned)wgs), 512, 0, s>>>(t, (const uint16_t *)Q, (uint16_t *)O, LSE, p.N,
                                                                           wgs);
    } else {                                          // d = 128: one query block per wave (registers), 8 per workgroup
        const int64_t wgs = (int64_t)p.bh * (p.N / 128);
        attn_fwd_shared_kernel<128, 1><<<dim3((unsigned)wgs), 512, 0, s>>>(t, (const uint16_t *)Q, (uint16_t *)O, LSE,
                                                                            p.N, wgs);
    }
    return hipGetLastError();
}

}  // namespace llsa
