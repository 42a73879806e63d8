// dK, dV of the gathered-list attention on bf16 MFMA (B = 16, d = 64 or 128), Sec. 4.3: key-major over
// the transposed lists of Alg. 2 (or over every query at the coarsest enriched level), with no mask and
// no floating-point atomics.
// With P = exp(z - LSE), dP = dO V^T, dS = P o (dP - D):  dK = scale dS^T Q,  dV = P^T dO.
//
// One workgroup (4 waves) per (key block of 16 level-l tokens, split).  The queries that attend to the
// block are the fine queries under the level-l query blocks listed for it, walked in groups of 16
// consecutive queries; a tile is two groups.  The tiles of the workgroup's share are dealt round-robin
// to its waves.  Per tile:
//   S = Q K^T, dP = dO V^T   (lane: 4 queries x 1 key)  ->  P, dS  ->
//   dV^T += dO^T P,  dK^T += Q^T dS   (A = the Q / dO tile read transposed from LDS, B = P / dS).
// The four waves' accumulators are summed through LDS in wave order, so the result does not depend on
// timing.  Level 0 (no split) finishes in place: adds the parent token's share (adjoint of mean pooling)
// and rounds once; coarser levels write fp32 partial sums, one slab per split, that a second kernel
// adds up in split order.
#include "mfma_common.h"

namespace llsa {

struct DkvArgs {
    const uint16_t *Q, *dO, *Kl, *Vl;     // Kl, Vl: the level's keys / values [bh, n_l, D]
    const float *LSE, *Dsum;
    const int32_t *C, *Iq;                // key-major lists (unused when dense)
    float *partK, *partV;                 // [splits][slab] fp32 (levels >= 1)
    const float *parK, *parV;             // level-1 totals [bh, n_1, D] fp32 or null (level 0)
    uint16_t *dK, *dV;                    // level-0 outputs
    int64_t N, n_l, rows, slab;           // rows = key blocks of this level per head that have lists
    int span_shift;                       // log2 of the 16-query groups per listed query block = 4 * level
    int Kl_cnt, level, dense, splits;
    float sc2, bias2, scale;
};

template <int D>
__global__ void __launch_bounds__(256) dkv_mfma_kernel(DkvArgs a) {
    constexpr int KS = D / 32, NT = D / 16, STRIDE = D * 2 + 32, VCH = D / 16, PARTS = D / 8, KPU = 64 / PARTS;
    constexpr int TILE = 32 * STRIDE;
    __shared__ __attribute__((aligned(16))) char lds[4][2 * TILE];   // per wave: Q tile | dO tile

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t nkb = (a.n_l + 15) >> 4;                 // key blocks per head
    const int64_t kbf = blockIdx.x / a.splits;             // flat key block
    const int split = blockIdx.x % a.splits;
    const int64_t bh = kbf / nkb, j = kbf % nkb;
    const int cntk = (int)min((int64_t)16, a.n_l - j * 16);
    char *qt = lds[wave], *gt = lds[wave] + TILE;

    // this block's keys and values: B operands (columns = keys), held for the whole kernel
    bf16x8 kop[KS], vop[KS];
    {
        const int64_t row = bh * a.n_l + j * 16 + min(i16, cntk - 1);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            kop[s] = ld_bf16x8(a.Kl + row * D + g * 8 + 32 * s);
            vop[s] = ld_bf16x8(a.Vl + row * D + g * 8 + 32 * s);
        }
    }
    // the 16-query groups of this key block
    const int32_t *lst = nullptr;
    int64_t groups;
    if (a.dense) {
        groups = a.N >> 4;
    } else {
        const int32_t *Crow = a.C + bh * (a.rows + 1) + j;
        const int32_t beg = Crow[0], end = Crow[1];
        lst = a.Iq + bh * a.rows * a.Kl_cnt + beg;
        groups = (int64_t)(end - beg) << a.span_shift;
    }
    const int64_t tiles = (groups + 1) >> 1;
    const int64_t t_beg = tiles * split / a.splits, t_end = tiles * (split + 1) / a.splits;
    const int64_t span_mask = ((int64_t)1 << a.span_shift) - 1;

    f32x4 accK[NT], accV[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) { accK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }

    int voff[VCH];
#pragma unroll
    for (int u = 0; u < VCH; ++u) voff[u] = (((lane / PARTS + KPU * u) & 15) * D + (lane % PARTS) * 8) * 2;

    u32x4 qreg[VCH], greg[VCH];
    f32x4 lse[2], del[2];
    int valid1;                                             // does the tile have its second group?
    auto load_tile = [&](int64_t tile) {
        const char *qp[2], *gp[2];
        valid1 = 2 * tile + 1 < groups;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t gi = (h == 0 || valid1) ? 2 * tile + h : 2 * tile;   // an absent group re-reads the first
            const int64_t q0 = a.dense ? gi * 16 : (((int64_t)lst[gi >> a.span_shift] << a.span_shift) + (gi & span_mask)) * 16;
            const int64_t row0 = bh * a.N + q0;
            lse[h] = *reinterpret_cast<const f32x4 *>(a.LSE + row0 + 4 * g);
            del[h] = *reinterpret_cast<const f32x4 *>(a.Dsum + row0 + 4 * g);
            qp[h] = reinterpret_cast<const char *>(a.Q + row0 * D);
            gp[h] = reinterpret_cast<const char *>(a.dO + row0 * D);
        }
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            const int h = (KPU * u) >> 4;
            qreg[u] = *reinterpret_cast<const u32x4 *>(qp[h] + voff[u]);
            greg[u] = *reinterpret_cast<const u32x4 *>(gp[h] + voff[u]);
        }
    };

    int64_t tile = t_beg + wave;
    if (tile < t_end) load_tile(tile);
    while (tile < t_end) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            const int q = lane / PARTS + KPU * u, part = lane % PARTS;
            *reinterpret_cast<u32x4 *>(qt + q * STRIDE + part * 16) = qreg[u];
            *reinterpret_cast<u32x4 *>(gt + q * STRIDE + part * 16) = greg[u];
        }
        __builtin_amdgcn_wave_barrier();

        f32x4 s[2], dp[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
            dp[h] = f32x4{0.f, 0.f, 0.f, 0.f};
            const char *qrow = qt + (h * 16 + i16) * STRIDE + g * 16, *grow = gt + (h * 16 + i16) * STRIDE + g * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s[h] = mfma16(*reinterpret_cast<const bf16x8 *>(qrow + ks * 64), kop[ks], s[h]);
                dp[h] = mfma16(*reinterpret_cast<const bf16x8 *>(grow + ks * 64), vop[ks], dp[h]);
            }
        }
        const f32x4 l2[2] = {lse[0], lse[1]}, dl[2] = {del[0], del[1]};
        const int v1 = valid1;
        const int64_t next = tile + 4;
        if (next < t_end) load_tile(next);

#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[h][r], a.sc2, fmaf(l2[h][r], -kLog2e, a.bias2)));
                s[h][r] = p;
                dp[h][r] = p * (dp[h][r] - dl[h][r]);
            }
        if (!v1) {                                          // the list ends with a single group
            s[1] = f32x4{0.f, 0.f, 0.f, 0.f};
            dp[1] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const bf16x8 pop = pack8(s[0], s[1]), dsop = pack8(dp[0], dp[1]);
        const int boff = (4 * g + (i16 >> 2)) * STRIDE + (i16 & 3) * 8;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            accV[n] = mfma16(lds_tr_pair(gt + boff + n * 32, gt + boff + 16 * STRIDE + n * 32), pop, accV[n]);
            accK[n] = mfma16(lds_tr_pair(qt + boff + n * 32, qt + boff + 16 * STRIDE + n * 32), dsop, accK[n]);
        }
        tile = next;
    }

    // sum the four waves' accumulators in wave order through LDS (reusing the tile buffers)
    __syncthreads();
    float *red = reinterpret_cast<float *>(&lds[0][0]);     // [wave][2 * NT][64 lanes] float4 slots
    constexpr int SLOTS = 2 * NT;
    static_assert(4 * SLOTS * 64 * 16 <= 4 * 2 * TILE, "reduction buffer must fit in the tile buffers");
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        *reinterpret_cast<f32x4 *>(red + ((wave * SLOTS + n) * 64 + lane) * 4) = accK[n];
        *reinterpret_cast<f32x4 *>(red + ((wave * SLOTS + NT + n) * 64 + lane) * 4) = accV[n];
    }
    __syncthreads();
    // wave w finishes slots w, w+4, ...: slot = which * NT + n
    for (int slot = wave; slot < SLOTS; slot += 4) {
        f32x4 sum = *reinterpret_cast<const f32x4 *>(red + ((0 * SLOTS + slot) * 64 + lane) * 4);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(red + ((w * SLOTS + slot) * 64 + lane) * 4);
#pragma unroll
            for (int r = 0; r < 4; ++r) sum[r] += x[r];
        }
        const bool isV = slot >= NT;
        const int n = isV ? slot - NT : slot;
        if (i16 >= cntk) continue;                          // rows past the end of a ragged coarsest level
        const int64_t tok = bh * a.n_l + j * 16 + i16;
        const int col = n * 16 + 4 * g;                     // lane holds 4 consecutive channels of key i16
        if (!isV)
#pragma unroll
            for (int r = 0; r < 4; ++r) sum[r] *= a.scale;
        if (a.level > 0) {
            float *dst = (isV ? a.partV : a.partK) + (int64_t)split * a.slab;
            *reinterpret_cast<f32x4 *>(dst + tok * D + col) = sum;
        } else {
            const float *par = isV ? a.parV : a.parK;
            if (par) {
                const f32x4 pv = *reinterpret_cast<const f32x4 *>(par + (bh * (a.n_l >> 4) + j) * D + col);
#pragma unroll
                for (int r = 0; r < 4; ++r) sum[r] += pv[r] * 0.0625f;
            }
            u32x2 w;
            w[0] = pack_bf16(sum[0], sum[1]);
            w[1] = pack_bf16(sum[2], sum[3]);
            *reinterpret_cast<u32x2 *>((isV ? a.dV : a.dK) + tok * D + col) = w;
        }
    }
}

// Adds the split slabs of one coarse level in split order and, if there is a coarser level above it,
// that level's share (adjoint of mean pooling, 1/16 of the parent token): dst[t] = sum_s part[s][t]
// (+ up[t / 16] / 16).  dst is the level's fp32 gradient buffer.  One thread per 4 consecutive floats.
__global__ void __launch_bounds__(256) dkv_reduce_kernel(const float *partK, const float *partV, float *dstK,
                                                          float *dstV, const float *upK, const float *upV,
                                                          int64_t total4, int64_t slab, int splits, int d) {
    const int64_t i4 = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i4 >= total4) return;
    const int64_t i = i4 * 4;
    f32x4 k = {0.f, 0.f, 0.f, 0.f}, v = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < splits; ++s) {
        k += *reinterpret_cast<const f32x4 *>(partK + s * slab + i);
        v += *reinterpret_cast<const f32x4 *>(partV + s * slab + i);
    }
    if (upK) {
        const int64_t tok = i / d, c = i % d;
        k += *reinterpret_cast<const f32x4 *>(upK + (tok >> 4) * d + c) * 0.0625f;
        v += *reinterpret_cast<const f32x4 *>(upV + (tok >> 4) * d + c) * 0.0625f;
    }
    *reinterpret_cast<f32x4 *>(dstK + i) = k;
    *reinterpret_cast<f32x4 *>(dstV + i) = v;
}

int dkv_splits(const Plan &p, int l) {
    if (l == 0) return 1;
    // aim for a few thousand workgroups per level; a workgroup should still see several tiles
    const int64_t key_blocks = (int64_t)p.bh * ((p.n[l] + 15) / 16);
    const int64_t tiles_per_block = (l == p.L) ? p.N / 32 : (int64_t)p.K * (p.N / p.n[l + 1]) / 32;  // average
    int64_t s = (4096 + key_blocks - 1) / key_blocks;
    if (s > tiles_per_block / 8) s = tiles_per_block / 8;
    if (s < 1) s = 1;
    if (s > 64) s = 64;
    return (int)s;
}

hipError_t launch_dkv_mfma(const Plan &p, const LevelTable &t, int l, const void *Q, const void *dO, const float *LSE,
                           const float *D, void *ws, void *dK, void *dV, hipStream_t s) {
    char *w = static_cast<char *>(ws);
    DkvArgs a;
    const int64_t key_blocks = (int64_t)p.bh * ((p.n[l] + 15) / 16);
    a.Q = (const uint16_t *)Q; a.dO = (const uint16_t *)dO;
    a.Kl = (const uint16_t *)t.K[l]; a.Vl = (const uint16_t *)t.V[l];
    a.LSE = LSE; a.Dsum = D;
    a.dense = (l == p.L);
    a.C = a.dense ? nullptr : (const int32_t *)(w + p.C_off[l]);
    a.Iq = a.dense ? nullptr : (const int32_t *)(w + p.Iq_off[l]);
    a.splits = dkv_splits(p, l);
    a.slab = key_blocks * 16 * p.d;
    a.partK = (float *)(w + p.part_off);
    a.partV = a.partK + (size_t)a.splits * a.slab;
    const bool has_parent = (l == 0 && p.Le >= 1);
    a.parK = has_parent ? (const float *)(w + p.dKacc_off[1]) : nullptr;
    a.parV = has_parent ? (const float *)(w + p.dVacc_off[1]) : nullptr;
    a.dK = (uint16_t *)dK; a.dV = (uint16_t *)dV;
    a.N = p.N; a.n_l = p.n[l];
    a.rows = a.dense ? 0 : p.n[l + 1];
    a.span_shift = a.dense ? 0 : 4 * l;
    a.Kl_cnt = a.dense ? 0 : p.Kl[l];
    a.level = l;
    a.sc2 = p.scale * kLog2e; a.bias2 = t.bias[l] * kLog2e; a.scale = p.scale;
    dim3 grid((unsigned)(key_blocks * a.splits));
    if (p.d == 64) dkv_mfma_kernel<64><<<grid, 256, 0, s>>>(a);
    else dkv_mfma_kernel<128><<<grid, 256, 0, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || l == 0) return e;
    // fold the slabs (and the level above) into this level's fp32 gradient
    const int64_t total4 = (int64_t)p.bh * p.n[l] * p.d / 4;
    const bool has_up = l < p.Le;
    dkv_reduce_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, s>>>(
        a.partK, a.partV, (float *)(w + p.dKacc_off[l]), (float *)(w + p.dVacc_off[l]),
        has_up ? (const float *)(w + p.dKacc_off[l + 1]) : nullptr, has_up ? (const float *)(w + p.dVacc_off[l + 1]) : nullptr,
        total4, a.slab, a.splits, p.d);
    return hipGetLastError();
}

}  // namespace llsa
