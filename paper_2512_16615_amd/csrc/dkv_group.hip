// dK, dV of the coarse levels (l >= 1) on bf16 MFMA, grouped by query block (B = 16, d = 64, N % 256 == 0).
//
// The 256 fine queries under one level-1 query block R attend to the same coarse key blocks (Alg. 1,
// enrichment loop: fine block i reads row i / B^l of I^(l)).  Key-major processing (Sec. 4.3) re-reads the
// Q / dO rows of R once per listed key block; here a workgroup stages them once in LDS and its 8 waves run
// the key-major tile loop over the 8 query tiles of R against R's coarse key blocks:
//   S = Q K^T, dP = dO V^T (lane: 4 queries x 1 key) -> P, dS -> dV^T += dO^T P, dK^T += Q^T dS.
// That yields, per (query group, coarse block of its list), the block's gradient restricted to the group's
// queries: an 8 KB fp32 partial.  Two kernels produce the partials:
//   dkv_group_kernel: one R per workgroup, every wave takes some of R's key blocks (any levels);
//   dkv_upper_kernel: levels >= 2 only.  The 16 level-1 blocks under one level-2 query block list the same
//     key blocks at every level >= 2, so a workgroup walks G of them (G divides 16) and keeps its
//     accumulators in registers meanwhile: every wave owns one or two of the listed key blocks, and the
//     single block of the coarsest level is shared (wave w takes query tile w of every R; the 8 waves'
//     sums are added through LDS at the end).  G times fewer partials, and none of the idle rounds the
//     first kernel has when the number of key blocks is not a multiple of 8.
// The partials are then added up in a fixed order:
//   1. levels l >= 2: the query groups under one level-l query block list the same key blocks, so their
//      partials are summed up to 16 at a time (slab_reduce_kernel) until one partial per level-l query
//      block is left; the coarsest enriched level (every query attends to it) is summed down to one
//      partial per head;
//   2. per level, top-down, every key block gathers the partials of the query blocks that listed it
//      (Alg. 2's key-major lists, ascending), adds the share of its parent token (adjoint of mean
//      pooling) and writes the level's fp32 gradient (dkv_gather_kernel).
// No floating-point atomics; every sum has a fixed order.
#include "mfma_common.h"

namespace llsa {

constexpr int kUnit = 2 * 16 * 64;                      // floats of one partial: [dK | dV][16 keys][64 channels]

struct GroupArgs {
    const uint16_t *Q, *dO;
    const float *LSE, *Dsum;
    float *slab;                                        // partials, level-major
    int64_t lvl_off[kMaxL + 1];                         // float offset of level l's partials [group][pos][kUnit]
    int nblk[kMaxL + 1];                                // key blocks of level l in a list
    int64_t N, NR;                                      // NR = level-1 query blocks per head
    int lev_end;                                        // levels below lev_end are processed (from 1, or from 2 in the upper kernel)
    int G;                                              // level-1 query blocks per workgroup (upper kernel)
    int nbs, nbd;                                       // upper kernel: listed blocks of its sparse levels / of the dense level
    float sc2, scale;
};

// ---- the staged group: 256 rows of Q and of dO, 128 bytes each, 16-byte chunks XOR-swizzled by row
__device__ __forceinline__ int swz(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }

struct StageRegs { u32x4 q[4], g[4]; float s; };

__device__ __forceinline__ void stage_load(StageRegs &r, const GroupArgs &a, int64_t row0, int tid) {
    const char *qsrc = reinterpret_cast<const char *>(a.Q + row0 * 64), *gsrc = reinterpret_cast<const char *>(a.dO + row0 * 64);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        r.q[k] = *reinterpret_cast<const u32x4 *>(qsrc + (tid + 512 * k) * 16);
        r.g[k] = *reinterpret_cast<const u32x4 *>(gsrc + (tid + 512 * k) * 16);
    }
    r.s = tid < 256 ? a.LSE[row0 + tid] : a.Dsum[row0 + tid - 256];
}
__device__ __forceinline__ void stage_store(const StageRegs &r, char *qs, char *gs, float *st, int tid) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int cc = tid + 512 * k;
        *reinterpret_cast<u32x4 *>(qs + swz(cc >> 3, cc & 7)) = r.q[k];
        *reinterpret_cast<u32x4 *>(gs + swz(cc >> 3, cc & 7)) = r.g[k];
    }
    st[tid] = r.s;                                      // LSE [256] | D [256]
}

// per-lane LDS offsets inside a 16-row slice (the swizzle key of a row depends only on the lane)
struct TileOffsets { int row[2], tr[4]; };
__device__ __forceinline__ TileOffsets tile_offsets(int lane) {
    const int i16 = lane & 15, g = lane >> 4;
    const int key_row = (i16 >> 1) & 7, key_tr = (2 * g + (i16 >> 3)) & 7;
    TileOffsets o;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) o.row[ks] = i16 * 128 + (((g + 4 * ks) ^ key_row) << 4);
#pragma unroll
    for (int n = 0; n < 4; ++n)
        o.tr[n] = (4 * g + (i16 >> 2)) * 128 + (((2 * n + ((i16 >> 1) & 1)) ^ key_tr) << 4) + ((i16 & 1) << 3);
    return o;
}

// queries 32u .. 32u+31 of the staged group against one block of 16 keys (kop / vop: its K / V rows as
// B operands): accK += Q^T dS, accV += dO^T P
__device__ __forceinline__ void group_tile(const char *qs, const char *gs, const float *st, int u, const TileOffsets &o,
                                           const bf16x8 (&kop)[2], const bf16x8 (&vop)[2], float bias2, float sc2,
                                           f32x4 (&accK)[4], f32x4 (&accV)[4], int g) {
    f32x4 s[2], dp[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int base = (32 * u + 16 * h) * 128;
        s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
        dp[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            s[h] = mfma16(*reinterpret_cast<const bf16x8 *>(qs + base + o.row[ks]), kop[ks], s[h]);
            dp[h] = mfma16(*reinterpret_cast<const bf16x8 *>(gs + base + o.row[ks]), vop[ks], dp[h]);
        }
        const f32x4 l2 = *reinterpret_cast<const f32x4 *>(st + 32 * u + 16 * h + 4 * g);
        const f32x4 dl = *reinterpret_cast<const f32x4 *>(st + 256 + 32 * u + 16 * h + 4 * g);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p = __builtin_amdgcn_exp2f(fmaf(s[h][r], sc2, fmaf(l2[r], -kLog2e, bias2)));
            s[h][r] = p;
            dp[h][r] = p * (dp[h][r] - dl[r]);
        }
    }
    const bf16x8 pop = pack8(s[0], s[1]), dsop = pack8(dp[0], dp[1]);
    const int b0 = 32 * u * 128, b1 = b0 + 16 * 128;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        accV[n] = mfma16(lds_tr_pair(gs + b0 + o.tr[n], gs + b1 + o.tr[n]), pop, accV[n]);
        accK[n] = mfma16(lds_tr_pair(qs + b0 + o.tr[n], qs + b1 + o.tr[n]), dsop, accK[n]);
    }
}

// K / V rows of one listed block as B operands (rows past a ragged end re-read the last row)
__device__ __forceinline__ void load_block_ops(const char *kp, const char *vp, int cnt, int lane, bf16x8 (&kop)[2],
                                               bf16x8 (&vop)[2]) {
    const int off = (min(lane & 15, cnt - 1) * 64 + (lane >> 4) * 8) * 2;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        kop[ks] = ld_bf16x8(kp + off + 64 * ks);
        vop[ks] = ld_bf16x8(vp + off + 64 * ks);
    }
}

// where the partial of list block jl (counted from the start of the list) of query group `grp` goes
__device__ __forceinline__ float *partial_ptr(const LevelTable &t, const GroupArgs &a, int nlev, int jl, int64_t grp) {
    int l = 1;
#pragma unroll
    for (int x = 2; x <= kMaxL; ++x) l += (x < nlev && jl >= t.bseg[x]) ? 1 : 0;
    const int pos = jl - pick(t.bseg, l);
    return a.slab + pick(a.lvl_off, l) + (grp * pick(a.nblk, l) + pos) * kUnit;
}

__device__ __forceinline__ void store_partial(float *dst, const f32x4 (&accK)[4], const f32x4 (&accV)[4], float scale, int lane) {
    dst += (lane & 15) * 64 + 4 * (lane >> 4);
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        f32x4 k = accK[n];
#pragma unroll
        for (int r = 0; r < 4; ++r) k[r] *= scale;
        *reinterpret_cast<f32x4 *>(dst + n * 16) = k;
        *reinterpret_cast<f32x4 *>(dst + 16 * 64 + n * 16) = accV[n];
    }
}

__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4)))
dkv_group_kernel(LevelTable t, GroupArgs a) {
    constexpr int D = 64;
    __shared__ __attribute__((aligned(16))) char qs[256 * 128];       // Q rows of the group, chunk-swizzled
    __shared__ __attribute__((aligned(16))) char gs[256 * 128];       // dO rows
    __shared__ __attribute__((aligned(16))) float st[512];            // LSE | D

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;
    const int64_t R = xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t bh = R / a.NR, Rh = R % a.NR;
    {
        StageRegs sr;
        stage_load(sr, a, bh * a.N + Rh * 256, tid);
        stage_store(sr, qs, gs, st, tid);
    }
    __syncthreads();
    const TileOffsets o = tile_offsets(lane);

    const int nlev = min(t.nlev, a.lev_end);
    const int c_begin = t.bseg[1], nbc = pick(t.bseg, nlev) - c_begin;
    BlockTable ctab;
    int chunk = -1;
    for (int jb = wave; jb < nbc; jb += 8) {
        if ((jb >> 6) != chunk) { chunk = jb >> 6; ctab.fill(t, bh, Rh * 16, c_begin, chunk, lane, D, nlev); }
        bf16x8 kop[2], vop[2];
        load_block_ops(ctab.K(jb & 63), ctab.V(jb & 63), ctab.count(jb & 63), lane, kop, vop);
        const float bias2 = ctab.bias(jb & 63);
        f32x4 accK[4], accV[4];
#pragma unroll
        for (int n = 0; n < 4; ++n) { accK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }
        for (int u = 0; u < 8; ++u) group_tile(qs, gs, st, u, o, kop, vop, bias2, a.sc2, accK, accV, g);
        store_partial(partial_ptr(t, a, nlev, jb + c_begin, R), accK, accV, a.scale, lane);
    }
}

// SS = listed sparse blocks a wave may own (blocks wave, wave + 8, ...)
template <int SS>
__global__ void __launch_bounds__(512) dkv_upper_kernel(LevelTable t, GroupArgs a) {
    constexpr int D = 64;
    __shared__ __attribute__((aligned(16))) char lds[2 * 256 * 128];  // Q rows | dO rows; the final reduction reuses it
    __shared__ __attribute__((aligned(16))) float st[512];
    char *qs = lds, *gs = lds + 256 * 128;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t per_head = a.NR / a.G;
    const int64_t grp = blockIdx.x;                                   // query group: G consecutive level-1 query blocks
    const int64_t bh = grp / per_head, R0 = (grp % per_head) * a.G;
    const TileOffsets o = tile_offsets(lane);

    const int nlev = min(t.nlev, a.lev_end);
    const int u_begin = t.bseg[2];                                    // first listed block of level 2
    BlockTable ctab;                                                  // lane j: listed block u_begin + j (at most 17)
    ctab.fill(t, bh, R0 * 16, u_begin, 0, lane, D, nlev);

    bf16x8 kopS[SS][2], vopS[SS][2], kopD[2], vopD[2];
    float biasS[SS], biasD = 0.f;
    f32x4 accSK[SS][4], accSV[SS][4], accDK[4], accDV[4];
#pragma unroll
    for (int s = 0; s < SS; ++s) {
        const int jb = wave + 8 * s;
        biasS[s] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) { kopS[s][ks] = bf16x8{}; vopS[s][ks] = bf16x8{}; }
        if (jb < a.nbs) {
            load_block_ops(ctab.K(jb), ctab.V(jb), 16, lane, kopS[s], vopS[s]);
            biasS[s] = ctab.bias(jb);
        }
#pragma unroll
        for (int n = 0; n < 4; ++n) { accSK[s][n] = f32x4{0.f, 0.f, 0.f, 0.f}; accSV[s][n] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) { kopD[ks] = bf16x8{}; vopD[ks] = bf16x8{}; }
    if (a.nbd) {
        load_block_ops(ctab.K(a.nbs), ctab.V(a.nbs), ctab.count(a.nbs), lane, kopD, vopD);
        biasD = ctab.bias(a.nbs);
    }
#pragma unroll
    for (int n = 0; n < 4; ++n) { accDK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accDV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }

    StageRegs sr;
    stage_load(sr, a, bh * a.N + R0 * 256, tid);
    for (int r = 0; r < a.G; ++r) {
        stage_store(sr, qs, gs, st, tid);
        __syncthreads();
        if (r + 1 < a.G) stage_load(sr, a, bh * a.N + (R0 + r + 1) * 256, tid);   // flies during the math
#pragma unroll
        for (int s = 0; s < SS; ++s)
            if (wave + 8 * s < a.nbs)
                for (int u = 0; u < 8; ++u) group_tile(qs, gs, st, u, o, kopS[s], vopS[s], biasS[s], a.sc2, accSK[s], accSV[s], g);
        if (a.nbd) group_tile(qs, gs, st, wave, o, kopD, vopD, biasD, a.sc2, accDK, accDV, g);
        __syncthreads();                                              // everyone is done with this R's rows
    }

#pragma unroll
    for (int s = 0; s < SS; ++s)
        if (wave + 8 * s < a.nbs)
            store_partial(partial_ptr(t, a, nlev, u_begin + wave + 8 * s, grp), accSK[s], accSV[s], a.scale, lane);
    if (a.nbd) {                                                      // the shared block: add the 8 waves' sums in wave order
        float *red = reinterpret_cast<float *>(lds);                  // [wave][slot][lane] f32x4, 64 KB
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            *reinterpret_cast<f32x4 *>(red + ((wave * 8 + n) * 64 + lane) * 4) = accDK[n];
            *reinterpret_cast<f32x4 *>(red + ((wave * 8 + 4 + n) * 64 + lane) * 4) = accDV[n];
        }
        __syncthreads();
        f32x4 sum = *reinterpret_cast<const f32x4 *>(red + (wave * 64 + lane) * 4);      // wave w owns slot w
#pragma unroll
        for (int w = 1; w < 8; ++w) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(red + ((w * 8 + wave) * 64 + lane) * 4);
#pragma unroll
            for (int c = 0; c < 4; ++c) sum[c] += x[c];
        }
        const bool isV = wave >= 4;
        if (!isV)
#pragma unroll
            for (int c = 0; c < 4; ++c) sum[c] *= a.scale;
        float *dst = partial_ptr(t, a, nlev, u_begin + a.nbs, grp) + (isV ? 16 * 64 : 0) + i16 * 64 + (wave & 3) * 16 + 4 * g;
        *reinterpret_cast<f32x4 *>(dst) = sum;
    }
}

// out[h][r][x] = sum_{c < f, f r + c < cnt_in} in[h][f r + c][x], x over `width` floats (one thread per float4)
__global__ void __launch_bounds__(256) slab_reduce_kernel(const float *in, float *out, int64_t cnt_in, int64_t cnt_out,
                                                           int64_t f, int64_t width4, int64_t total4) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total4) return;
    const int64_t x = i % width4, hr = i / width4, r = hr % cnt_out, h = hr / cnt_out;
    const int64_t first = f * r, n = min(f, cnt_in - first);
    const f32x4 *src = reinterpret_cast<const f32x4 *>(in) + (h * cnt_in + first) * width4 + x;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int64_t c = 0; c < n; ++c) acc += src[c * width4];
    reinterpret_cast<f32x4 *>(out)[i] = acc;
}

// One workgroup per key block j of level l: sums the partials of the query blocks that listed j, in list
// order, adds the parent token's share and writes the level's fp32 gradient rows.
struct GatherArgs {
    const float *part;           // [bh][cnt][nblk][kUnit]
    const int32_t *C, *Iq, *I;   // key-major lists and I^(l) (null when dense)
    const float *upK, *upV;      // gradient of level l + 1 or null
    float *dstK, *dstV;          // [bh, n_l, 64]
    int64_t cnt, n_l, nkb, rows; // listers per head, tokens, key blocks per head, rows of I^(l)
    int nblk, Kl, dense;
};
__global__ void __launch_bounds__(256) dkv_gather_kernel(GatherArgs a) {
    const int tid = threadIdx.x;
    const int64_t bh = blockIdx.x / a.nkb, j = blockIdx.x % a.nkb;
    const f32x4 *part = reinterpret_cast<const f32x4 *>(a.part);
    f32x4 k = {0.f, 0.f, 0.f, 0.f}, v = {0.f, 0.f, 0.f, 0.f};
    if (a.dense) {
        const f32x4 *p = part + ((bh * a.cnt) * a.nblk + j) * (kUnit / 4);
        k = p[tid];
        v = p[256 + tid];
    } else {
        // first every thread resolves one lister (query block row and the position of j in that row's list),
        // 256 at a time, then all threads add the partials in list order with independent loads
        __shared__ int64_t unit[256];
        const int32_t beg = a.C[bh * (a.rows + 1) + j], end = a.C[bh * (a.rows + 1) + j + 1];
        const int32_t *lst = a.Iq + bh * a.rows * a.Kl;
        for (int32_t e0 = beg; e0 < end; e0 += 256) {
            const int32_t m = min(256, end - e0);
            __syncthreads();
            if (tid < m) {
                const int64_t r = lst[e0 + tid];
                const int32_t *row = a.I + (bh * a.rows + r) * a.Kl;
                int pos = 0;
                for (int x = 0; x < a.Kl; ++x) pos += (row[x] < (int32_t)j) ? 1 : 0;   // rows are ascending
                unit[tid] = ((bh * a.cnt + r) * a.nblk + pos) * (kUnit / 4);
            }
            __syncthreads();
#pragma unroll 4
            for (int32_t e = 0; e < m; ++e) {
                const f32x4 *p = part + unit[e];
                k += p[tid];
                v += p[256 + tid];
            }
        }
    }
    const int64_t tok = j * 16 + (tid >> 4);
    if (tok >= a.n_l) return;
    const int col = (tid & 15) * 4;
    if (a.upK) {
        const int64_t up = (bh * ((a.n_l + 15) / 16) + j) * 64 + col;   // parent token of the block's 16 tokens
        k += *reinterpret_cast<const f32x4 *>(a.upK + up) * 0.0625f;
        v += *reinterpret_cast<const f32x4 *>(a.upV + up) * 0.0625f;
    }
    *reinterpret_cast<f32x4 *>(a.dstK + (bh * a.n_l + tok) * 64 + col) = k;
    *reinterpret_cast<f32x4 *>(a.dstV + (bh * a.n_l + tok) * 64 + col) = v;
}

// Highest level the grouped kernels take; levels above it go to the split key-major kernel.  Only a wide dense
// coarsest level is left out: every query block would write a partial sum for every one of its key blocks, and
// summing over all queries is what the split kernel does in registers.  (Sending a coarsest level of a single
// key block to the split kernel, to spare the 8 waves a third round for one block, was measured slower.)
int dkv_group_top(const Plan &p) {
    if (p.Le == p.L && (p.n[p.L] + 15) / 16 > 32) return p.L - 1;
    return p.Le;
}

// Listed blocks of levels 2 .. top: sparse levels (nbs) and the dense coarsest level (nbd).
static void upper_blocks(const Plan &p, int *nbs, int *nbd) {
    const int top = dkv_group_top(p);
    *nbs = *nbd = 0;
    for (int l = 2; l <= top; ++l) {
        if (l < p.L) *nbs += p.Kl[l];
        else *nbd = (int)((p.n[l] + 15) / 16);
    }
}

// Level-1 query blocks per workgroup of the upper kernel, or 0 if levels >= 2 stay with dkv_group_kernel:
// at most 16 sparse blocks (two per wave), at most one dense block.
static int upper_G(const Plan &p) {
    int nbs, nbd;
    upper_blocks(p, &nbs, &nbd);
    if (dkv_group_top(p) < 2 || nbs + nbd == 0 || nbs > 16 || nbd > 1) return 0;
    const int64_t NR = p.N / 256;
    int G = 16;                                             // divides 16, so a group never straddles a level-2 query block
    while (G > 1 && (NR % G != 0 || (int64_t)p.bh * (NR / G) < 256)) G >>= 1;
    return G;
}

// partial-slab layout: level 1 has one partial per (level-1 query block, list position), levels >= 2 one per
// (query group, list position)
static int64_t slab_layout(const Plan &p, int64_t *lvl_off, int *nblk, int64_t *groups) {
    const int64_t NR = p.N / 256;
    const int G = upper_G(p);
    int64_t off = 0;
    for (int l = 0; l <= kMaxL; ++l) { lvl_off[l] = 0; nblk[l] = 0; groups[l] = 0; }
    for (int l = 1; l <= dkv_group_top(p); ++l) {
        nblk[l] = l < p.L ? p.Kl[l] : (int)((p.n[l] + 15) / 16);
        groups[l] = (l >= 2 && G) ? NR / G : NR;
        lvl_off[l] = off;
        off += (int64_t)p.bh * groups[l] * nblk[l] * kUnit;
    }
    return off;
}

// bytes of the partial slab and of each of the two reduction buffers
void dkv_group_sizes(const Plan &p, size_t *slab_bytes, size_t *red_bytes) {
    const int64_t NR = p.N / 256;
    int64_t lvl_off[kMaxL + 1], groups[kMaxL + 1];
    int nblk[kMaxL + 1];
    *slab_bytes = (size_t)slab_layout(p, lvl_off, nblk, groups) * sizeof(float);
    size_t red = 0;
    for (int l = 1; l <= dkv_group_top(p); ++l) {
        const size_t r = (size_t)p.bh * ((NR + 15) / 16) * nblk[l] * kUnit * sizeof(float);
        if ((l >= 2 || l == p.L) && r > red) red = r;       // levels that get reduced before the gather
    }
    *red_bytes = red;
}

hipError_t launch_dkv_group(const Plan &p, const LevelTable &t, const void *Q, const void *dO, const float *LSE,
                            const float *D, void *ws, hipStream_t s) {
    char *w = static_cast<char *>(ws);
    const int64_t NR = p.N / 256;
    const int top = dkv_group_top(p), G = upper_G(p);
    GroupArgs a;
    int64_t groups[kMaxL + 1];
    a.Q = (const uint16_t *)Q; a.dO = (const uint16_t *)dO; a.LSE = LSE; a.Dsum = D;
    a.slab = (float *)(w + p.grp_slab_off);
    a.N = p.N; a.NR = NR;
    a.sc2 = p.scale * kLog2e; a.scale = p.scale;
    slab_layout(p, a.lvl_off, a.nblk, groups);
    a.G = G;
    upper_blocks(p, &a.nbs, &a.nbd);

    a.lev_end = G ? 2 : top + 1;
    dkv_group_kernel<<<dim3((unsigned)(p.bh * NR)), 512, 0, s>>>(t, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (G) {
        a.lev_end = top + 1;
        const dim3 grid((unsigned)(p.bh * (NR / G)));
        if (a.nbs > 8) dkv_upper_kernel<2><<<grid, 512, 0, s>>>(t, a);
        else dkv_upper_kernel<1><<<grid, 512, 0, s>>>(t, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }

    float *red[2] = {(float *)(w + p.grp_red_off[0]), (float *)(w + p.grp_red_off[1])};
    for (int l = top; l >= 1; --l) {                        // top-down: a level adds the share of the one above
        const bool dense = (l == p.L);
        const float *cur = a.slab + a.lvl_off[l];
        int64_t cnt = groups[l];
        const int64_t target = dense ? 1 : p.n[l + 1];      // listers per head: level-l query blocks, or the head
        const int64_t width4 = (int64_t)a.nblk[l] * (kUnit / 4);
        int flip = 0;
        while (cnt > target) {
            // groups under one lister are consecutive and their number is a power of two (any count when dense)
            const int64_t f = dense ? 16 : (cnt / target < 16 ? cnt / target : 16);
            const int64_t cnt_out = (cnt + f - 1) / f;
            const int64_t total4 = (int64_t)p.bh * cnt_out * width4;
            slab_reduce_kernel<<<dim3((unsigned)((total4 + 255) / 256)), 256, 0, s>>>(cur, red[flip], cnt, cnt_out, f, width4,
                                                                                      total4);
            cur = red[flip];
            flip ^= 1;
            cnt = cnt_out;
        }
        GatherArgs ga;
        ga.part = cur;
        ga.dense = dense;
        ga.C = dense ? nullptr : (const int32_t *)(w + p.C_off[l]);
        ga.Iq = dense ? nullptr : (const int32_t *)(w + p.Iq_off[l]);
        ga.I = dense ? nullptr : t.I[l];
        const bool has_up = l < p.Le;
        ga.upK = has_up ? (const float *)(w + p.dKacc_off[l + 1]) : nullptr;
        ga.upV = has_up ? (const float *)(w + p.dVacc_off[l + 1]) : nullptr;
        ga.dstK = (float *)(w + p.dKacc_off[l]);
        ga.dstV = (float *)(w + p.dVacc_off[l]);
        ga.cnt = cnt; ga.n_l = p.n[l]; ga.nkb = (p.n[l] + 15) / 16; ga.rows = dense ? 0 : p.n[l + 1];
        ga.nblk = a.nblk[l]; ga.Kl = dense ? 0 : p.Kl[l];
        dkv_gather_kernel<<<dim3((unsigned)(p.bh * ga.nkb)), 256, 0, s>>>(ga);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace llsa
