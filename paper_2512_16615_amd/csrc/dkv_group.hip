// dK, dV of the coarse levels (l >= 1) on bf16 MFMA, grouped by query block (B = 16, d = 64, N % 256 == 0).
//
// The 256 fine queries under one level-1 query block R attend to the same coarse key blocks (Alg. 1,
// enrichment loop: fine block i reads row i / B^l of I^(l)).  Key-major processing (Sec. 4.3) re-reads the
// Q / dO rows of R once per listed key block; here a workgroup stages them once in LDS and its waves run
// the key-major tile loop over the 8 query tiles of R against R's coarse key blocks:
//   S = Q K^T, dP = dO V^T (lane: 4 queries x 1 key) -> P, dS -> dV^T += dO^T P, dK^T += Q^T dS.
// That yields, per (query group, coarse block of its list), the block's gradient restricted to the group's
// queries: an 8 KB fp32 partial.  Two kernels produce the partials:
//   dkv_group_kernel: one R per workgroup of 4 waves; wave w takes list blocks 2w, 2w+1 (then 2w+8, ... if
//     the list is longer) of the levels it is given and feeds both from one LDS read of each tile;
//   dkv_upper_kernel: levels >= 2 only.  The 16 level-1 blocks under one level-2 query block list the same
//     key blocks at every level >= 2, so a workgroup of 8 waves walks G of them (G divides 16; the next one's
//     rows are prefetched into registers) and keeps its accumulators in registers meanwhile: every wave owns
//     one or two of the listed blocks (16 per launch), and the single block of the coarsest level is shared
//     (wave w takes query tile w of every R; the 8 waves' sums are added through LDS at the end).  G times
//     fewer partials, and no idle rounds when the number of key blocks is not a multiple of the waves.
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
    int sparse_begin, do_dense;                         // upper kernel: first sparse block of this launch; does it take the dense one
    float sc2, scale;
};

// ---- the staged group: 256 rows of Q and of dO, 128 bytes each (half a row of the 64 LDS banks), 16-byte
// chunks XOR-swizzled by row.  The key gives the 16 rows of a slice 8 distinct values per row parity, so the
// row-wise 16-byte reads of 16 lanes hit 16 different bank groups.  (A key that also spreads the transposed
// 8-byte reads of a half wave was timed: those reads did not get faster, the row-wise ones got slower.)
__device__ __forceinline__ int swz_key(int r) { return (r >> 1) & 7; }
__device__ __forceinline__ int swz(int r, int c) { return r * 128 + ((c ^ swz_key(r)) << 4); }

// 256 threads copy the 256 Q and dO rows starting at row0, and their LSE and D, into LDS
__device__ __forceinline__ void stage_rows(const GroupArgs &a, int64_t row0, char *qs, char *gs, float *st, int tid) {
    const char *qsrc = reinterpret_cast<const char *>(a.Q + row0 * 64), *gsrc = reinterpret_cast<const char *>(a.dO + row0 * 64);
    u32x4 q[8], g[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        q[k] = *reinterpret_cast<const u32x4 *>(qsrc + (tid + 256 * k) * 16);
        g[k] = *reinterpret_cast<const u32x4 *>(gsrc + (tid + 256 * k) * 16);
    }
    const float l = a.LSE[row0 + tid], d = a.Dsum[row0 + tid];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int cc = tid + 256 * k;
        *reinterpret_cast<u32x4 *>(qs + swz(cc >> 3, cc & 7)) = q[k];
        *reinterpret_cast<u32x4 *>(gs + swz(cc >> 3, cc & 7)) = g[k];
    }
    st[tid] = l;                                        // LSE [256] | D [256]
    st[256 + tid] = d;
}

// per-lane LDS offsets inside a 16-row slice (the swizzle key of a row depends only on the lane)
struct TileOffsets { int row[2], tr[4]; };
__device__ __forceinline__ TileOffsets tile_offsets(int lane) {
    const int i16 = lane & 15, g = lane >> 4;
    const int key_row = swz_key(i16), key_tr = swz_key(4 * g + (i16 >> 2));   // rows of a slice: i16 resp. 4g + i16 / 4
    TileOffsets o;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) o.row[ks] = i16 * 128 + (((g + 4 * ks) ^ key_row) << 4);
#pragma unroll
    for (int n = 0; n < 4; ++n)
        o.tr[n] = (4 * g + (i16 >> 2)) * 128 + (((2 * n + ((i16 >> 1) & 1)) ^ key_tr) << 4) + ((i16 & 1) << 3);
    return o;
}

// One key block held by a wave: its K / V rows as B operands, the level's log2 weight, its gradient sums.
struct BlockAcc {
    bf16x8 kop[2], vop[2];
    float bias2;
    f32x4 accK[4], accV[4];

    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int n = 0; n < 4; ++n) { accK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    }
    // rows past a ragged end re-read the last row; an absent block (kp = null) gets zero operands
    __device__ __forceinline__ void load(const char *kp, const char *vp, int cnt, float b2, int lane) {
        bias2 = b2;
        const int off = (min(lane & 15, max(cnt, 1) - 1) * 64 + (lane >> 4) * 8) * 2;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            kop[ks] = kp ? ld_bf16x8(kp + off + 64 * ks) : bf16x8{};
            vop[ks] = kp ? ld_bf16x8(vp + off + 64 * ks) : bf16x8{};
        }
    }
};

// queries 32u .. 32u+31 of the staged group against NB key blocks: accK += Q^T dS, accV += dO^T P.
// Every LDS operand is read once and used for all NB blocks.
template <int NB>
__device__ __forceinline__ void group_tile(const char *qs, const char *gs, const float *st, int u, const TileOffsets &o,
                                           BlockAcc (&blk)[NB], float sc2, int g) {
    f32x4 s[NB][2], dp[NB][2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int base = (32 * u + 16 * h) * 128;
        bf16x8 aq[2], ag[2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            aq[ks] = *reinterpret_cast<const bf16x8 *>(qs + base + o.row[ks]);
            ag[ks] = *reinterpret_cast<const bf16x8 *>(gs + base + o.row[ks]);
        }
        const f32x4 l2 = *reinterpret_cast<const f32x4 *>(st + 32 * u + 16 * h + 4 * g);
        const f32x4 dl = *reinterpret_cast<const f32x4 *>(st + 256 + 32 * u + 16 * h + 4 * g);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            s[b][h] = f32x4{0.f, 0.f, 0.f, 0.f};
            dp[b][h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                s[b][h] = mfma16(aq[ks], blk[b].kop[ks], s[b][h]);
                dp[b][h] = mfma16(ag[ks], blk[b].vop[ks], dp[b][h]);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[b][h][r], sc2, fmaf(l2[r], -kLog2e, blk[b].bias2)));
                s[b][h][r] = p;
                dp[b][h][r] = p * (dp[b][h][r] - dl[r]);
            }
        }
    }
    bf16x8 pop[NB], dsop[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) { pop[b] = pack8(s[b][0], s[b][1]); dsop[b] = pack8(dp[b][0], dp[b][1]); }
    const int b0 = 32 * u * 128, b1 = b0 + 16 * 128;
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        const bf16x8 tg = lds_tr_pair(gs + b0 + o.tr[n], gs + b1 + o.tr[n]);
        const bf16x8 tq = lds_tr_pair(qs + b0 + o.tr[n], qs + b1 + o.tr[n]);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            blk[b].accV[n] = mfma16(tg, pop[b], blk[b].accV[n]);
            blk[b].accK[n] = mfma16(tq, dsop[b], blk[b].accK[n]);
        }
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

__device__ __forceinline__ void store_partial(float *dst, const BlockAcc &b, float scale, int lane) {
    dst += (lane & 15) * 64 + 4 * (lane >> 4);
#pragma unroll
    for (int n = 0; n < 4; ++n) {
        f32x4 k = b.accK[n];
#pragma unroll
        for (int r = 0; r < 4; ++r) k[r] *= scale;
        *reinterpret_cast<f32x4 *>(dst + n * 16) = k;
        *reinterpret_cast<f32x4 *>(dst + 16 * 64 + n * 16) = b.accV[n];
    }
}

__global__ void __launch_bounds__(256) dkv_group_kernel(LevelTable t, GroupArgs a) {
    constexpr int D = 64;
    __shared__ __attribute__((aligned(16))) char qs[256 * 128];       // Q rows of the group, chunk-swizzled
    __shared__ __attribute__((aligned(16))) char gs[256 * 128];       // dO rows
    __shared__ __attribute__((aligned(16))) float st[512];            // LSE | D

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;
    const int64_t R = xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t bh = R / a.NR, Rh = R % a.NR;
    stage_rows(a, bh * a.N + Rh * 256, qs, gs, st, tid);
    __syncthreads();
    const TileOffsets o = tile_offsets(lane);

    const int nlev = min(t.nlev, a.lev_end);
    const int c_begin = t.bseg[1], nbc = pick(t.bseg, nlev) - c_begin;
    BlockTable ctab;
    int chunk = -1;
    for (int jb = 2 * wave; jb < nbc; jb += 8) {                      // blocks jb, jb + 1 (same chunk of 64: jb is even)
        if ((jb >> 6) != chunk) { chunk = jb >> 6; ctab.fill(t, bh, Rh * 16, c_begin, chunk, lane, D, nlev); }
        const bool two = jb + 1 < nbc;
        BlockAcc blk[2];
        blk[0].load(ctab.K(jb & 63), ctab.V(jb & 63), ctab.count(jb & 63), ctab.bias(jb & 63), lane);
        blk[1].load(two ? ctab.K((jb + 1) & 63) : nullptr, ctab.V((jb + 1) & 63), ctab.count((jb + 1) & 63),
                    ctab.bias((jb + 1) & 63), lane);
        blk[0].clear();
        blk[1].clear();
        for (int u = 0; u < 8; ++u) group_tile<2>(qs, gs, st, u, o, blk, a.sc2, g);
        store_partial(partial_ptr(t, a, nlev, jb + c_begin, R), blk[0], a.scale, lane);
        if (two) store_partial(partial_ptr(t, a, nlev, jb + 1 + c_begin, R), blk[1], a.scale, lane);
    }
}

// 512 threads: the same copy split in two, so that the loads of the next group can fly during the math
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
    st[tid] = r.s;
}

// SS = sparse blocks a wave owns in one launch (blocks sparse_begin + wave, + 8, ...): a launch covers 8 SS of them
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
    BlockAcc sp[SS][1], dn[1];                                        // this wave's sparse blocks; the dense block
    {
        BlockTable ctab;                                              // lane j: listed block u_begin + 64 * chunk + j
        int chunk = -1;
#pragma unroll
        for (int s = 0; s < SS; ++s) {
            const int jb = a.sparse_begin + wave + 8 * s;
            const bool have = jb < a.nbs;
            if (have && (jb >> 6) != chunk) { chunk = jb >> 6; ctab.fill(t, bh, R0 * 16, u_begin, chunk, lane, D, nlev); }
            sp[s][0].load(have ? ctab.K(jb & 63) : nullptr, ctab.V(jb & 63), 16, ctab.bias(jb & 63), lane);
            sp[s][0].clear();
        }
        if (a.do_dense) {
            if ((a.nbs >> 6) != chunk) ctab.fill(t, bh, R0 * 16, u_begin, a.nbs >> 6, lane, D, nlev);
            dn[0].load(ctab.K(a.nbs & 63), ctab.V(a.nbs & 63), ctab.count(a.nbs & 63), ctab.bias(a.nbs & 63), lane);
        } else {
            dn[0].load(nullptr, nullptr, 16, 0.f, lane);
        }
        dn[0].clear();
    }

    StageRegs sr;
    stage_load(sr, a, bh * a.N + R0 * 256, tid);
    for (int r = 0; r < a.G; ++r) {
        stage_store(sr, qs, gs, st, tid);
        __syncthreads();
        if (r + 1 < a.G) stage_load(sr, a, bh * a.N + (R0 + r + 1) * 256, tid);   // flies during the math
#pragma unroll
        for (int s = 0; s < SS; ++s)
            if (a.sparse_begin + wave + 8 * s < a.nbs)
                for (int u = 0; u < 8; ++u) group_tile<1>(qs, gs, st, u, o, sp[s], a.sc2, g);
        if (a.do_dense) group_tile<1>(qs, gs, st, wave, o, dn, a.sc2, g);
        __syncthreads();                                              // everyone is done with this R's rows
    }

#pragma unroll
    for (int s = 0; s < SS; ++s) {
        const int jb = a.sparse_begin + wave + 8 * s;
        if (jb < a.nbs) store_partial(partial_ptr(t, a, nlev, u_begin + jb, grp), sp[s][0], a.scale, lane);
    }
    if (a.do_dense) {                                                 // the shared block: add the 8 waves' sums in wave order
        float *red = reinterpret_cast<float *>(lds);                  // [wave][slot][lane] f32x4, 64 KB
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            *reinterpret_cast<f32x4 *>(red + ((wave * 8 + n) * 64 + lane) * 4) = dn[0].accK[n];
            *reinterpret_cast<f32x4 *>(red + ((wave * 8 + 4 + n) * 64 + lane) * 4) = dn[0].accV[n];
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
// summing over all queries is what the split kernel does in registers.
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

// Level-1 query blocks per workgroup of the upper kernel, or 0 if levels >= 2 stay with dkv_group_kernel
// (a dense level of more than one block).
static int upper_G(const Plan &p) {
    int nbs, nbd;
    upper_blocks(p, &nbs, &nbd);
    if (dkv_group_top(p) < 2 || nbs + nbd == 0 || nbd > 1) return 0;
    const int64_t NR = p.N / 256;
    int G = 16;                                             // divides 16, so a group never straddles a level-2 query block
    while (G > 1 && (NR % G != 0 || (int64_t)p.bh * (NR / G) < 256)) G >>= 1;  // one workgroup of 8 waves per CU
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

#define GRP_TRY(expr)                     \
    do {                                  \
        const hipError_t e_ = (expr);     \
        if (e_ != hipSuccess) return e_;  \
    } while (0)

// reductions and gather of level l on stream s; `groups` = partials per head the kernels left for the level
static hipError_t finish_level(const Plan &p, const LevelTable &t, const GroupArgs &a, int l, int64_t groups, char *w,
                               hipStream_t s) {
    float *red[2] = {(float *)(w + p.grp_red_off[0]), (float *)(w + p.grp_red_off[1])};
    const bool dense = (l == p.L);
    const float *cur = a.slab + a.lvl_off[l];
    int64_t cnt = groups;
    const int64_t target = dense ? 1 : p.n[l + 1];          // listers per head: level-l query blocks, or the head
    const int64_t width4 = (int64_t)a.nblk[l] * (kUnit / 4);
    int flip = 0;
    while (cnt > target) {
        // groups under one lister are consecutive and their number is a power of two (any count when dense)
        const int64_t f = dense ? 16 : (cnt / target < 16 ? cnt / target : 16);
        const int64_t cnt_out = (cnt + f - 1) / f;
        const int64_t total4 = (int64_t)p.bh * cnt_out * width4;
        slab_reduce_kernel<<<dim3((unsigned)((total4 + 255) / 256)), 256, 0, s>>>(cur, red[flip], cnt, cnt_out, f, width4, total4);
        GRP_TRY(hipGetLastError());
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
    return hipGetLastError();
}

hipError_t launch_dkv_group(const Plan &p, const LevelTable &t, const void *Q, const void *dO, const float *LSE,
                            const float *D, void *ws, hipStream_t s, hipStream_t side, hipEvent_t ev_fork,
                            hipEvent_t ev_join) {
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
    a.sparse_begin = 0;
    a.do_dense = 0;

    if (!G) {                                               // one kernel for every level, then top-down (a level adds the share of the one above)
        a.lev_end = top + 1;
        dkv_group_kernel<<<dim3((unsigned)(p.bh * NR)), 256, 0, s>>>(t, a);
        GRP_TRY(hipGetLastError());
        for (int l = top; l >= 1; --l) GRP_TRY(finish_level(p, t, a, l, groups[l], w, s));
        return hipSuccess;
    }

    // levels >= 2 (their own kernel, reductions and gathers, which share the two reduction buffers) beside level 1's kernel
    const bool fork = side != s;
    if (fork) {
        GRP_TRY(hipEventRecord(ev_fork, s));
        GRP_TRY(hipStreamWaitEvent(side, ev_fork, 0));
    }
    GroupArgs up = a;
    up.lev_end = top + 1;
    const dim3 grid((unsigned)(p.bh * (NR / G)));
    for (int sb = 0; sb == 0 || sb < up.nbs; sb += 16) {    // up to 16 sparse blocks per launch; the first also takes the dense one
        up.sparse_begin = sb;
        up.do_dense = (sb == 0 && up.nbd > 0) ? 1 : 0;
        if (up.nbs - sb > 8) dkv_upper_kernel<2><<<grid, 512, 0, side>>>(t, up);
        else dkv_upper_kernel<1><<<grid, 512, 0, side>>>(t, up);
        GRP_TRY(hipGetLastError());
    }
    for (int l = top; l >= 2; --l) GRP_TRY(finish_level(p, t, up, l, groups[l], w, side));
    if (fork) GRP_TRY(hipEventRecord(ev_join, side));

    a.lev_end = 2;
    dkv_group_kernel<<<dim3((unsigned)(p.bh * NR)), 256, 0, s>>>(t, a);
    GRP_TRY(hipGetLastError());
    if (fork) GRP_TRY(hipStreamWaitEvent(s, ev_join, 0));
    return finish_level(p, t, a, 1, groups[1], w, s);     // level 1 has no reduction, so the buffers are free of a race
}

}  // namespace llsa
