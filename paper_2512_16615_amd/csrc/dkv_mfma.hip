// dK, dV of the gathered-list attention on bf16 MFMA (B = 16, 32 or 64, d = 64 or 128), Sec. 4.3: key-major over
// the transposed lists of Alg. 2 (or over every query at the coarsest enriched level), with no mask and
// no floating-point atomics.
// With P = exp(z - LSE), dP = dO V^T, dS = P o (dP - D):  dK = scale dS^T Q,  dV = P^T dO.
//
// The unit of work is a tile of 16 level-l keys (a listed block of B keys is B / 16 tiles with one list).  The
// queries that attend to it are the fine queries under the level-l query blocks listed for its block, walked in
// groups of 16 consecutive queries; a tile of the loop is two groups.  Per tile a wave
// computes
//   S = Q K^T, dP = dO V^T   (lane: 4 queries x 1 key)  ->  P, dS  ->
//   dV^T += dO^T P,  dK^T += Q^T dS   (A = the Q / dO tile read transposed from LDS, B = P / dS).
// Two kernels share that tile loop:
//   dkv_coarse_kernel (levels >= 1): one workgroup of 4 waves per (key block, split); the tiles of its
//     share are dealt round-robin to the waves, whose accumulators are summed through LDS in wave order;
//     fp32 partial sums go to one slab per split and a second kernel adds the slabs in split order (and
//     the share of the level above, the adjoint of mean pooling).
//   dkv_fine_kernel (level 0): lists are short (K on average), so every wave takes one key block of its
//     own; a key block whose list is long is instead worked on by all four waves together afterwards.
//     The epilogue adds the parent token's share and rounds once to bf16.
// Every sum has a fixed order, so results do not depend on timing.
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
    int span_shift;                       // log2 of the 16-query groups per listed query block: log2(B^(level+1) / 16)
    int ls, lb;                           // log2(B / 16), log2 B: 16-key tile j lies in listed block j >> ls
    float inv_B;
    int Kl_cnt, dense, splits;
    float sc2, bias2, scale;
};

template <int D> struct DkvShape {
    static constexpr int KS = D / 32, NT = D / 16, STRIDE = D * 2 + 32, VCH = D / 16, PARTS = D / 8, KPU = 64 / PARTS;
    static constexpr int TILE = 32 * STRIDE;
};

// Tiles t_first, t_first + t_step, ... < t_end of one key block's query list, accumulated into accK / accV.
// lst: the block's listed query-block rows (null when dense); groups: 16-query groups in the list.
template <int D>
__device__ __forceinline__ void dkv_tile_loop(const DkvArgs &a, int64_t bh, const int32_t *lst, int64_t groups,
                                              int64_t t_first, int64_t t_step, int64_t t_end,
                                              const bf16x8 (&kop)[D / 32], const bf16x8 (&vop)[D / 32],
                                              f32x4 (&accK)[D / 16], f32x4 (&accV)[D / 16], char *qt, char *gt,
                                              int lane) {
    using S = DkvShape<D>;
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t span_mask = ((int64_t)1 << a.span_shift) - 1;
    const int64_t entries = groups >> a.span_shift;
    unsigned voff[S::VCH];
#pragma unroll
    for (int u = 0; u < S::VCH; ++u) voff[u] = (unsigned)((((lane / S::PARTS + S::KPU * u) & 15) * D + (lane % S::PARTS) * 8) * 2);

    // the list entries, 64 at a time in one register (lane e: entry 64 * chunk + e)
    int ecache = 0;
    int64_t echunk = -1;
    auto entry = [&](int64_t e) -> int64_t {
        if ((e >> 6) != echunk) {
            echunk = e >> 6;
            const int64_t idx = echunk * 64 + lane;
            ecache = idx < entries ? lst[idx] : 0;
        }
        return __builtin_amdgcn_readlane(ecache, (int)(e & 63));
    };

    u32x4 qreg[S::VCH], greg[S::VCH];
    float stat = 0.f;                                       // lane x: LSE (x < 32) or D (x >= 32) of tile query x % 32
    int valid1 = 0;                                         // does the tile have its second group?
    float *st = reinterpret_cast<float *>(gt + S::TILE);    // 64 floats behind the two tiles
    auto load_tile = [&](int64_t tile) {
        const char *qp[2], *gp[2];
        valid1 = 2 * tile + 1 < groups;
        int64_t row0[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t gi = (h == 0 || valid1) ? 2 * tile + h : 2 * tile;   // an absent group re-reads the first
            const int64_t q0 = a.dense ? gi * 16 : ((entry(gi >> a.span_shift) << a.span_shift) + (gi & span_mask)) * 16;
            row0[h] = bh * a.N + q0;
            qp[h] = reinterpret_cast<const char *>(a.Q + row0[h] * D);
            gp[h] = reinterpret_cast<const char *>(a.dO + row0[h] * D);
        }
        stat = ((lane & 32) ? a.Dsum : a.LSE)[((lane & 16) ? row0[1] : row0[0]) + i16];
#pragma unroll
        for (int u = 0; u < S::VCH; ++u) {
            const int h = (S::KPU * u) >> 4;
            qreg[u] = *reinterpret_cast<const u32x4 *>(qp[h] + voff[u]);
            greg[u] = *reinterpret_cast<const u32x4 *>(gp[h] + voff[u]);
        }
    };

    int64_t tile = t_first;
    if (tile < t_end) load_tile(tile);
    while (tile < t_end) {
        __builtin_amdgcn_wave_barrier();                    // one wave's LDS operations stay in order
#pragma unroll
        for (int u = 0; u < S::VCH; ++u) {
            const int q = lane / S::PARTS + S::KPU * u, part = lane % S::PARTS;
            *reinterpret_cast<u32x4 *>(qt + q * S::STRIDE + part * 16) = qreg[u];
            *reinterpret_cast<u32x4 *>(gt + q * S::STRIDE + part * 16) = greg[u];
        }
        st[lane] = stat;
        __builtin_amdgcn_wave_barrier();

        f32x4 s[2], dp[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
            dp[h] = f32x4{0.f, 0.f, 0.f, 0.f};
            const char *qrow = qt + (h * 16 + i16) * S::STRIDE + g * 16, *grow = gt + (h * 16 + i16) * S::STRIDE + g * 16;
#pragma unroll
            for (int ks = 0; ks < S::KS; ++ks) {
                s[h] = mfma16(*reinterpret_cast<const bf16x8 *>(qrow + ks * 64), kop[ks], s[h]);
                dp[h] = mfma16(*reinterpret_cast<const bf16x8 *>(grow + ks * 64), vop[ks], dp[h]);
            }
        }
        // this lane's 4 queries per half: rows 4g .. 4g+3
        const f32x4 l2[2] = {*reinterpret_cast<const f32x4 *>(st + 4 * g), *reinterpret_cast<const f32x4 *>(st + 16 + 4 * g)};
        const f32x4 dl[2] = {*reinterpret_cast<const f32x4 *>(st + 32 + 4 * g),
                             *reinterpret_cast<const f32x4 *>(st + 48 + 4 * g)};
        const int v1 = valid1;
        const int64_t next = tile + t_step;
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
        const int boff = (4 * g + (i16 >> 2)) * S::STRIDE + (i16 & 3) * 8;
#pragma unroll
        for (int n = 0; n < S::NT; ++n) {
            accV[n] = mfma16(lds_tr_pair(gt + boff + n * 32, gt + boff + 16 * S::STRIDE + n * 32), pop, accV[n]);
            accK[n] = mfma16(lds_tr_pair(qt + boff + n * 32, qt + boff + 16 * S::STRIDE + n * 32), dsop, accK[n]);
        }
        tile = next;
    }
}

// Sum of the four waves' accumulators in wave order through LDS; wave w ends up owning slots w, w + 4, ...
// (slot = which * NT + n, which: 0 = dK, 1 = dV) and hands each finished slot to `emit(slot, sum)`.
template <int D, class Emit>
__device__ __forceinline__ void dkv_reduce_waves(float *red, int wave, int lane, const f32x4 (&accK)[D / 16],
                                                 const f32x4 (&accV)[D / 16], Emit emit) {
    constexpr int NT = D / 16, SLOTS = 2 * NT;
    __syncthreads();                                        // everyone is done with the tile buffers
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        *reinterpret_cast<f32x4 *>(red + ((wave * SLOTS + n) * 64 + lane) * 4) = accK[n];
        *reinterpret_cast<f32x4 *>(red + ((wave * SLOTS + NT + n) * 64 + lane) * 4) = accV[n];
    }
    __syncthreads();
    for (int slot = wave; slot < SLOTS; slot += 4) {
        f32x4 sum = *reinterpret_cast<const f32x4 *>(red + ((0 * SLOTS + slot) * 64 + lane) * 4);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(red + ((w * SLOTS + slot) * 64 + lane) * 4);
#pragma unroll
            for (int r = 0; r < 4; ++r) sum[r] += x[r];
        }
        emit(slot, sum);
    }
}

template <int D>
__device__ __forceinline__ void dkv_load_keys(const DkvArgs &a, int64_t row, int lane, bf16x8 (&kop)[D / 32],
                                              bf16x8 (&vop)[D / 32]) {
    const int g = lane >> 4;
#pragma unroll
    for (int s = 0; s < D / 32; ++s) {
        kop[s] = ld_bf16x8(a.Kl + row * D + g * 8 + 32 * s);
        vop[s] = ld_bf16x8(a.Vl + row * D + g * 8 + 32 * s);
    }
}

// ----------------------------------------------------------------------------------------- levels >= 1
template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 3 : 2))) dkv_coarse_kernel(DkvArgs a) {
    using S = DkvShape<D>;
    __shared__ __attribute__((aligned(16))) char lds[4][2 * S::TILE + 256];   // per wave: Q tile | dO tile | LSE, D
    static_assert(4 * 2 * S::NT * 64 * 16 <= 4 * 2 * S::TILE, "reduction buffer must fit in the tile buffers");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t nkb = (a.n_l + 15) >> 4;                 // key blocks per head
    const int64_t wgid = xcd_contiguous(blockIdx.x, gridDim.x);   // neighbouring key blocks share query tiles in L2
    const int64_t kbf = wgid / a.splits;                   // flat key block
    const int split = (int)(wgid % a.splits);
    const int64_t bh = kbf / nkb, j = kbf % nkb;
    const int cntk = (int)min((int64_t)16, a.n_l - j * 16);

    bf16x8 kop[S::KS], vop[S::KS];                          // B operands (columns = keys), held throughout
    dkv_load_keys<D>(a, bh * a.n_l + j * 16 + min(i16, cntk - 1), lane, kop, vop);
    const int32_t *lst = nullptr;
    int64_t groups;
    if (a.dense) {
        groups = a.N >> 4;
    } else {
        const int32_t *Crow = a.C + bh * (a.rows + 1) + (j >> a.ls);
        const int32_t beg = Crow[0], end = Crow[1];
        lst = a.Iq + bh * a.rows * a.Kl_cnt + beg;
        groups = (int64_t)(end - beg) << a.span_shift;
    }
    const int64_t tiles = (groups + 1) >> 1;
    const int64_t t_beg = tiles * split / a.splits, t_end = tiles * (split + 1) / a.splits;

    f32x4 accK[S::NT], accV[S::NT];
#pragma unroll
    for (int n = 0; n < S::NT; ++n) { accK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    dkv_tile_loop<D>(a, bh, lst, groups, t_beg + wave, 4, t_end, kop, vop, accK, accV, lds[wave], lds[wave] + S::TILE, lane);

    dkv_reduce_waves<D>(reinterpret_cast<float *>(&lds[0][0]), wave, lane, accK, accV, [&](int slot, f32x4 sum) {
        const bool isV = slot >= S::NT;
        const int n = isV ? slot - S::NT : slot;
        if (i16 >= cntk) return;                            // rows past the end of a ragged coarsest level
        if (!isV)
#pragma unroll
            for (int r = 0; r < 4; ++r) sum[r] *= a.scale;
        float *dst = (isV ? a.partV : a.partK) + (int64_t)split * a.slab;
        *reinterpret_cast<f32x4 *>(dst + (bh * a.n_l + j * 16 + i16) * D + n * 16 + 4 * g) = sum;
    });
}

// ---------------------------------------------------------------------------------------------- level 0
constexpr int kSoloMax = 24;                                // longest list (16-query groups) one wave takes alone

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 3 : 2))) dkv_fine_kernel(DkvArgs a) {
    using S = DkvShape<D>;
    __shared__ __attribute__((aligned(16))) char lds[4][2 * S::TILE + 256];
    __shared__ int len_sh[4];
    __shared__ __attribute__((aligned(16))) float par_sh[4][2 * D];   // per wave: the parent token's dK | dV

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t nkb = a.n_l >> 4;                        // key blocks per head (a multiple of 4)
    const bool has_par = a.parK != nullptr;
    // The 16 key blocks under one level-1 token draw their queries from one pool (the fine blocks under the
    // level-1 query blocks that listed that token), about 0.5 MB of Q and dO.  Keep the four workgroups of
    // such a group on one XCD (ids congruent modulo 8) so the pool is fetched into one L2 only, and deal
    // the groups round-robin over the XCDs so that clusters of hot key blocks are spread.
    // (Measured: keeping such a group on one XCD does not pay; the plain order spreads hot clusters best.)
    const int64_t kb0 = (int64_t)blockIdx.x * 4;           // this workgroup's four key blocks (same head)
    const int64_t bh = kb0 / nkb;

    // The 16 keys of block j share one parent token (level-1 token j).  Its gradient row is fetched into
    // registers before the tile loop (so the epilogue does not wait for memory) and handed to the epilogue's
    // channel layout through the wave's LDS row.
    float park[D / 64], parv[D / 64];
    auto par_fetch = [&](int64_t j) {
#pragma unroll
        for (int x = 0; x < D / 64; ++x) {
            park[x] = has_par ? a.parK[(bh * (nkb >> a.ls) + (j >> a.ls)) * D + lane + 64 * x] : 0.f;
            parv[x] = has_par ? a.parV[(bh * (nkb >> a.ls) + (j >> a.ls)) * D + lane + 64 * x] : 0.f;
        }
    };
    auto par_publish = [&]() {                              // the wave's own row; its LDS operations stay in order
#pragma unroll
        for (int x = 0; x < D / 64; ++x) {
            par_sh[wave][lane + 64 * x] = park[x];
            par_sh[wave][D + lane + 64 * x] = parv[x];
        }
        __builtin_amdgcn_wave_barrier();
    };
    // level-0 epilogue: scale dK, add the parent token's share (adjoint of mean pooling), round once
    auto emit = [&](int64_t j, int slot, f32x4 sum) {
        const bool isV = slot >= S::NT;
        const int n = isV ? slot - S::NT : slot;
        const int col = n * 16 + 4 * g;                     // lane holds 4 consecutive channels of key i16
        if (!isV)
#pragma unroll
            for (int r = 0; r < 4; ++r) sum[r] *= a.scale;
        if (has_par) {
            const f32x4 pv = *reinterpret_cast<const f32x4 *>(&par_sh[wave][(isV ? D : 0) + col]);
#pragma unroll
            for (int r = 0; r < 4; ++r) sum[r] += pv[r] * a.inv_B;
        }
        u32x2 w;
        w[0] = pack_bf16(sum[0], sum[1]);
        w[1] = pack_bf16(sum[2], sum[3]);
        *reinterpret_cast<u32x2 *>((isV ? a.dV : a.dK) + (bh * a.n_l + j * 16 + i16) * D + col) = w;
    };

    // ---- each wave alone on its own key block, if that block's list is short
    {
        const int64_t j = kb0 % nkb + wave;
        const int32_t *Crow = a.C + bh * (a.rows + 1) + (j >> a.ls);
        const int32_t beg = Crow[0], len = (Crow[1] - beg) << a.span_shift;   // in 16-query groups
        if (lane == 0) len_sh[wave] = len;
        if (len <= kSoloMax) {
            bf16x8 kop[S::KS], vop[S::KS];
            f32x4 accK[S::NT], accV[S::NT];
            par_fetch(j);
#pragma unroll
            for (int n = 0; n < S::NT; ++n) { accK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }
            if (len > 0) {
                dkv_load_keys<D>(a, bh * a.n_l + j * 16 + i16, lane, kop, vop);
                dkv_tile_loop<D>(a, bh, a.Iq + bh * a.rows * a.Kl_cnt + beg, len, 0, 1, ((int64_t)len + 1) >> 1, kop, vop,
                                 accK, accV, lds[wave], lds[wave] + S::TILE, lane);
            }
            par_publish();
#pragma unroll
            for (int n = 0; n < S::NT; ++n) { emit(j, n, accK[n]); emit(j, S::NT + n, accV[n]); }
        }
    }
    __syncthreads();
    // ---- long lists: all four waves together, one key block after the other
    for (int w = 0; w < 4; ++w) {
        const int len = len_sh[w];
        if (len <= kSoloMax) continue;                      // uniform over the workgroup
        const int64_t j = kb0 % nkb + w;
        const int32_t beg = a.C[bh * (a.rows + 1) + (j >> a.ls)];
        bf16x8 kop[S::KS], vop[S::KS];
        f32x4 accK[S::NT], accV[S::NT];
#pragma unroll
        for (int n = 0; n < S::NT; ++n) { accK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        par_fetch(j);
        dkv_load_keys<D>(a, bh * a.n_l + j * 16 + i16, lane, kop, vop);
        dkv_tile_loop<D>(a, bh, a.Iq + bh * a.rows * a.Kl_cnt + beg, len, wave, 4, ((int64_t)len + 1) >> 1, kop, vop, accK,
                         accV, lds[wave], lds[wave] + S::TILE, lane);
        par_publish();
        dkv_reduce_waves<D>(reinterpret_cast<float *>(&lds[0][0]), wave, lane, accK, accV,
                            [&](int slot, f32x4 sum) { emit(j, slot, sum); });
        __syncthreads();                                    // the reduction buffer is the next round's tile space
    }
}

// Adds the split slabs of one coarse level in split order and, if there is a coarser level above it,
// that level's share (adjoint of mean pooling, 1/B of the parent token): dst[t] = sum_s part[s][t]
// (+ up[t / B] / B).  dst is the level's fp32 gradient buffer.  One thread per 4 consecutive floats.
__global__ void __launch_bounds__(256) dkv_reduce_kernel(const float *partK, const float *partV, float *dstK,
                                                          float *dstV, const float *upK, const float *upV,
                                                          int64_t total4, int64_t slab, int splits, int d, int lb,
                                                          float inv_B) {
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
        k += *reinterpret_cast<const f32x4 *>(upK + (tok >> lb) * d + c) * inv_B;
        v += *reinterpret_cast<const f32x4 *>(upV + (tok >> lb) * d + c) * inv_B;
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

// level0_alone: level 0's own gradient only, without the share of its parent tokens (the pooled levels' gradients)
hipError_t launch_dkv_mfma(const Plan &p, const LevelTable &t, int l, const void *Q, const void *dO, const float *LSE,
                           const float *D, void *ws, void *dK, void *dV, hipStream_t s, bool level0_alone) {
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
    const bool has_parent = (l == 0 && p.Le >= 1 && !level0_alone);
    a.parK = has_parent ? (const float *)(w + p.dKacc_off[1]) : nullptr;
    a.parV = has_parent ? (const float *)(w + p.dVacc_off[1]) : nullptr;
    a.dK = (uint16_t *)dK; a.dV = (uint16_t *)dV;
    a.N = p.N; a.n_l = p.n[l];
    a.rows = a.dense ? 0 : p.n[l + 1];
    a.span_shift = a.dense ? 0 : p.lb * (l + 1) - 4;
    a.ls = p.lb - 4; a.lb = p.lb; a.inv_B = 1.f / (float)p.B;
    a.Kl_cnt = a.dense ? 0 : p.Kl[l];
    a.sc2 = p.scale * kLog2e; a.bias2 = t.bias[l] * kLog2e; a.scale = p.scale;
    if (l == 0) {                                           // N % 64 == 0: four key blocks per workgroup, one head
        dim3 grid((unsigned)(key_blocks / 4));
        if (p.d == 64) dkv_fine_kernel<64><<<grid, 256, 0, s>>>(a);
        else dkv_fine_kernel<128><<<grid, 256, 0, s>>>(a);
        return hipGetLastError();
    }
    dim3 grid((unsigned)(key_blocks * a.splits));
    if (p.d == 64) dkv_coarse_kernel<64><<<grid, 256, 0, s>>>(a);
    else dkv_coarse_kernel<128><<<grid, 256, 0, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // fold the slabs (and the level above) into this level's fp32 gradient
    const int64_t total4 = (int64_t)p.bh * p.n[l] * p.d / 4;
    const bool has_up = l < p.Le;
    dkv_reduce_kernel<<<(unsigned)((total4 + 255) / 256), 256, 0, s>>>(
        a.partK, a.partV, (float *)(w + p.dKacc_off[l]), (float *)(w + p.dVacc_off[l]),
        has_up ? (const float *)(w + p.dKacc_off[l + 1]) : nullptr, has_up ? (const float *)(w + p.dVacc_off[l + 1]) : nullptr,
        total4, a.slab, a.splits, p.d, p.lb, 1.f / (float)p.B);
    return hipGetLastError();
}

}  // namespace llsa
