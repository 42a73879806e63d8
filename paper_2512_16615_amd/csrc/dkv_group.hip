// dK, dV of the coarse levels (l >= 1) on bf16 MFMA, grouped by query block (B = 16, d = 64 or 128, N % 256 == 0).
//
// The 256 fine queries under one level-1 query block R attend to the same coarse key blocks (Alg. 1,
// enrichment loop: fine block i reads row i / B^l of I^(l)).  Key-major processing (Sec. 4.3) re-reads the
// Q / dO rows of R once per listed key block; here a workgroup stages them once in LDS and its waves run
// the key-major tile loop over the 8 query tiles of R against R's coarse key blocks:
//   S = Q K^T, dP = dO V^T (lane: 4 queries x 1 key) -> P, dS -> dV^T += dO^T P, dK^T += Q^T dS.
// That yields, per (query group, coarse block of its list), the block's gradient restricted to the group's
// queries: a fp32 partial of 2 x 16 x d values.  Three kernels produce the partials:
//   dkv_group_kernel: one R per workgroup; a wave takes NB list blocks at a time (d = 64: 4 waves x 2 blocks fed
//     from one LDS read of each tile; d = 128: 8 waves x 1 block) of the levels it is given;
//   dkv_chain_kernel: level 1 with 8 listed blocks at d = 64.  The same tile loop, but a workgroup walks several
//     consecutive R and a key block listed by a run of them keeps its sums in registers: one partial per run;
//   dkv_upper_kernel: levels >= 2 only.  The 16 level-1 blocks under one level-2 query block list the same
//     key blocks at every level >= 2, so a workgroup of 8 waves walks G of them (G divides 16; the next one's
//     rows are prefetched into registers) and keeps its accumulators in registers meanwhile: every wave owns
//     one or two of the listed blocks, and (d = 64) the single block of the coarsest level is shared: wave w takes
//     query tile w of every R and the 8 waves' sums are added through LDS at the end.  G times fewer partials,
//     and no idle rounds when the number of key blocks is not a multiple of the waves.
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

template <int D> struct GShape {
    static constexpr int ROWB = 2 * D;                  // bytes of a staged row
    static constexpr int CH = D / 8;                    // 16-byte chunks per row
    static constexpr int KS = D / 32, NT = D / 16;
    static constexpr int UNIT = 2 * 16 * D;             // floats of one partial: [dK | dV][16 keys][D channels]
};

struct GroupArgs {
    const uint16_t *Q, *dO;
    const float *LSE, *Dsum;
    float *slab;                                        // partials, level-major
    int64_t lvl_off[kMaxL + 1];                         // float offset of level l's partials [group][pos][UNIT]
    int nblk[kMaxL + 1];                                // key blocks of level l in a list
    int64_t N, NR;                                      // NR = level-1 query blocks per head
    int lev_end;                                        // levels below lev_end are processed (from 1, or from 2 in the upper kernel)
    int G;                                              // level-1 query blocks per workgroup (upper kernel)
    int GC;                                             // level-1 query blocks a workgroup of the chain kernel walks
    int nbs, nbd;                                       // upper kernel: listed blocks of its sparse levels / of the dense level
    int sparse_begin, do_dense;                         // upper kernel: first sparse block of this launch; does it take the dense one
    float sc2, scale;
};

// ---- the staged group: 256 rows of Q and of dO, unpadded, 16-byte chunks XOR-swizzled by row (swz_key)
template <int D> __device__ __forceinline__ int swz(int r, int c) { return r * GShape<D>::ROWB + ((c ^ swz_key<D>(r)) << 4); }

// The 256 Q and dO rows from row0 on, and their LSE and D, in the registers of NTHR threads ...
template <int D, int NTHR> struct StageRegs {
    static constexpr int PER = 256 * GShape<D>::CH / NTHR;
    u32x4 q[PER], g[PER];
    float s[512 / NTHR];
};
template <int D, int NTHR>
__device__ __forceinline__ void stage_load(StageRegs<D, NTHR> &r, const GroupArgs &a, int64_t row0, int tid) {
    const char *qsrc = reinterpret_cast<const char *>(a.Q + row0 * D), *gsrc = reinterpret_cast<const char *>(a.dO + row0 * D);
#pragma unroll
    for (int k = 0; k < StageRegs<D, NTHR>::PER; ++k) {
        r.q[k] = *reinterpret_cast<const u32x4 *>(qsrc + (tid + NTHR * k) * 16);
        r.g[k] = *reinterpret_cast<const u32x4 *>(gsrc + (tid + NTHR * k) * 16);
    }
#pragma unroll
    for (int k = 0; k < 512 / NTHR; ++k) {
        const int i = tid + NTHR * k;
        r.s[k] = i < 256 ? a.LSE[row0 + i] : a.Dsum[row0 + i - 256];
    }
}
// ... and from there into LDS (qs, gs: swizzled rows; st: -LSE log2(e) [256] | D [256])
template <int D, int NTHR>
__device__ __forceinline__ void stage_store(const StageRegs<D, NTHR> &r, char *qs, char *gs, float *st, int tid) {
    constexpr int CH = GShape<D>::CH;
#pragma unroll
    for (int k = 0; k < StageRegs<D, NTHR>::PER; ++k) {
        const int cc = tid + NTHR * k;
        *reinterpret_cast<u32x4 *>(qs + swz<D>(cc / CH, cc % CH)) = r.q[k];
        *reinterpret_cast<u32x4 *>(gs + swz<D>(cc / CH, cc % CH)) = r.g[k];
    }
    // LSE goes in as -LSE log2(e), the form the tiles' exponentials take it in
#pragma unroll
    for (int k = 0; k < 512 / NTHR; ++k) st[tid + NTHR * k] = (tid + NTHR * k < 256) ? r.s[k] * -kLog2e : r.s[k];
}

// One key block held by a wave: its K / V rows as B operands, the level's log2 weight, its gradient sums.
// The tiles compute P = exp(z - LSE) without the level's weight B^l (a power of two for the block sizes of this
// path: scaling by it commutes with the bf16 rounding of P and dS); the sums take it when they are written.
template <int D> struct BlockAcc {
    bf16x8 kop[D / 32], vop[D / 32];
    float bias2;
    f32x4 accK[D / 16], accV[D / 16];

    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int n = 0; n < D / 16; ++n) { accK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    }
    // rows past a ragged end re-read the last row; an absent block (kp = null) gets zero operands
    __device__ __forceinline__ void load(const char *kp, const char *vp, int cnt, float b2, int lane) {
        bias2 = b2;
        const int off = (min(lane & 15, max(cnt, 1) - 1) * D + (lane >> 4) * 8) * 2;
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) {
            kop[ks] = kp ? ld_bf16x8(kp + off + 64 * ks) : bf16x8{};
            vop[ks] = kp ? ld_bf16x8(vp + off + 64 * ks) : bf16x8{};
        }
    }
};

// queries 32u .. 32u+31 of the staged group against NB key blocks: accK += Q^T dS, accV += dO^T P.
// Every LDS operand is read once and used for all NB blocks.
template <int D, int NB>
__device__ __forceinline__ void group_tile(const char *qs, const char *gs, const float *st, int u, const TileOffsets<D> &o,
                                           BlockAcc<D> (&blk)[NB], float sc2, int g) {
    using S = GShape<D>;
    f32x4 s[NB][2], dp[NB][2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int base = (32 * u + 16 * h) * S::ROWB;
        bf16x8 aq[S::KS], ag[S::KS];
#pragma unroll
        for (int ks = 0; ks < S::KS; ++ks) {
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
            for (int ks = 0; ks < S::KS; ++ks) {
                s[b][h] = mfma16(aq[ks], blk[b].kop[ks], s[b][h]);
                dp[b][h] = mfma16(ag[ks], blk[b].vop[ks], dp[b][h]);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[b][h][r], sc2, l2[r]));   // without the level's weight
                s[b][h][r] = p;
                dp[b][h][r] = p * (dp[b][h][r] - dl[r]);
            }
        }
    }
    bf16x8 pop[NB], dsop[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) { pop[b] = pack8(s[b][0], s[b][1]); dsop[b] = pack8(dp[b][0], dp[b][1]); }
    const int b0 = 32 * u * S::ROWB, b1 = b0 + 16 * S::ROWB;
#pragma unroll
    for (int n = 0; n < S::NT; ++n) {
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
template <int D>
__device__ __forceinline__ float *partial_ptr(const LevelTable &t, const GroupArgs &a, int nlev, int jl, int64_t grp) {
    int l = 1;
#pragma unroll
    for (int x = 2; x <= kMaxL; ++x) l += (x < nlev && jl >= t.bseg[x]) ? 1 : 0;
    const int pos = jl - pick(t.bseg, l);
    return a.slab + pick(a.lvl_off, l) + (grp * pick(a.nblk, l) + pos) * GShape<D>::UNIT;
}

template <int D> __device__ __forceinline__ void store_partial(float *dst, const BlockAcc<D> &b, float scale, int lane) {
    dst += (lane & 15) * D + 4 * (lane >> 4);
    const float w = __builtin_amdgcn_exp2f(b.bias2);        // the level's weight, left out of the tiles' P
    const float ws = w * scale;
#pragma unroll
    for (int n = 0; n < D / 16; ++n) {
        f32x4 k = b.accK[n], v = b.accV[n];
#pragma unroll
        for (int r = 0; r < 4; ++r) { k[r] *= ws; v[r] *= w; }
        *reinterpret_cast<f32x4 *>(dst + n * 16) = k;
        *reinterpret_cast<f32x4 *>(dst + 16 * D + n * 16) = v;
    }
}

// NW waves, NB key blocks per wave at a time
template <int D, int NW, int NB>
__global__ void __launch_bounds__(64 * NW) dkv_group_kernel(LevelTable t, GroupArgs a) {
    using S = GShape<D>;
    __shared__ __attribute__((aligned(16))) char qs[256 * S::ROWB];   // Q rows of the group, chunk-swizzled
    __shared__ __attribute__((aligned(16))) char gs[256 * S::ROWB];   // dO rows
    __shared__ __attribute__((aligned(16))) float st[512];            // LSE | D

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;
    const int64_t R = xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t bh = R / a.NR, Rh = R % a.NR;
    {
        StageRegs<D, 64 * NW> sr;
        stage_load<D, 64 * NW>(sr, a, bh * a.N + Rh * 256, tid);
        stage_store<D, 64 * NW>(sr, qs, gs, st, tid);
    }
    __syncthreads();
    const TileOffsets<D> o = tile_offsets<D>(lane);

    const int nlev = min(t.nlev, a.lev_end);
    const int c_begin = t.bseg[1], nbc = pick(t.bseg, nlev) - c_begin;
    BlockTable ctab;
    int chunk = -1;
    for (int jb = NB * wave; jb < nbc; jb += NB * NW) {               // blocks jb .. jb + NB - 1 (same chunk of 64: NB divides 64)
        if ((jb >> 6) != chunk) { chunk = jb >> 6; ctab.fill(t, bh, Rh * 16, c_begin, chunk, lane, D, nlev); }
        BlockAcc<D> blk[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int j = (jb + b) & 63;
            blk[b].load(jb + b < nbc ? ctab.K(j) : nullptr, ctab.V(j), ctab.count(j), ctab.bias(j), lane);
            blk[b].clear();
        }
        for (int u = 0; u < 8; ++u) group_tile<D, NB>(qs, gs, st, u, o, blk, a.sc2, g);
#pragma unroll
        for (int b = 0; b < NB; ++b)
            if (jb + b < nbc) store_partial<D>(partial_ptr<D>(t, a, nlev, jb + b + c_begin, R), blk[b], a.scale, lane);
    }
}

// Level 1 alone, rows of I^(1) with exactly NW * NB entries.  Neighbouring level-1 query blocks list mostly the same
// level-1 key blocks (for spatially smooth inputs a block stays listed over many consecutive rows), and a partial per
// (query block, listed block) then carries the same key block's sums to memory again and again.  Here a workgroup
// walks GC consecutive level-1 query blocks and keeps one listed block per register slot, as dkv_group_kernel does
// for a single query block.  From one query block R to the next, a slot whose key block is listed again goes on
// accumulating; a slot whose block is not listed by R + 1 writes its partial to the place of (R, the block's
// position in R's row) and takes one of the blocks that are new in R + 1 (both rows have NW * NB distinct entries,
// so as many slots come free as blocks are new).  A partial therefore covers a run of consecutive query blocks of
// one chain that all list the key block, and sits where the last of them would have put its own; the gather skips
// a lister whose successor in the same chain lists the block too.  Same arithmetic per tile, fewer partials.
template <int D, int NW, int NB>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) dkv_chain_kernel(LevelTable t, GroupArgs a) {
    using S = GShape<D>;
    constexpr int SL = NW * NB;
    __shared__ __attribute__((aligned(16))) char qs[256 * S::ROWB];
    __shared__ __attribute__((aligned(16))) char gs[256 * S::ROWB];
    __shared__ __attribute__((aligned(16))) float st[512];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4;
    const int64_t per_head = a.NR / a.GC;
    const int64_t grp = xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t bh = grp / per_head, R0 = (grp % per_head) * a.GC;
    const TileOffsets<D> o = tile_offsets<D>(lane);
    const int32_t *I1 = t.I[1] + (bh * a.NR + R0) * SL;               // I^(1) has one row per level-1 query block
    const char *K1 = static_cast<const char *>(t.K[1]) + bh * t.n[1] * D * 2;
    const char *V1 = static_cast<const char *>(t.V[1]) + bh * t.n[1] * D * 2;
    const float bias2 = t.bias[1] * kLog2e;
    float *slab1 = a.slab + a.lvl_off[1] + (bh * a.NR + R0) * SL * S::UNIT;

    int sblk = -1, spos = 0;                                          // lane s < SL: the block slot s holds, its place in the row
    BlockAcc<D> blk[NB];                                              // this wave's slots NB * wave ...
    for (int r = 0; r < a.GC; ++r) {
        StageRegs<D, 64 * NW> sr;
        stage_load<D, 64 * NW>(sr, a, bh * a.N + (R0 + r) * 256, tid);   // in flight during the bookkeeping below
        const int nb = lane < SL ? I1[r * SL + lane] : -1;            // lane p: entry p of this query block's row
        if (r == 0) {
            sblk = nb;
            spos = lane;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int64_t id = __builtin_amdgcn_readlane(nb, NB * wave + b);
                blk[b].load(K1 + id * 16 * D * 2, V1 + id * 16 * D * 2, 16, bias2, lane);
                blk[b].clear();
            }
        } else {
            bool keep = false, fresh = lane < SL;
            int npos = 0;
#pragma unroll
            for (int x = 0; x < SL; ++x) {
                if (sblk == __builtin_amdgcn_readlane(nb, x)) { keep = true; npos = x; }
                if (nb == __builtin_amdgcn_readlane(sblk, x)) fresh = false;
            }
            const uint64_t kept = __ballot(keep), freed = __ballot(lane < SL && !keep), news = __ballot(fresh);
            // the k-th slot that comes free takes the k-th new entry of the row
            const int k = __popcll(freed & ((1ull << lane) - 1));
            uint64_t m = news;
#pragma unroll
            for (int x = 0; x < SL; ++x) m = (x < k) ? (m & (m - 1)) : m;
            const int src = m ? (int)__builtin_ctzll(m) : 0;
            const int nid = __shfl(nb, src, 64);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int s = NB * wave + b;
                if (!((kept >> s) & 1)) {                             // wave-uniform
                    const int oldpos = __builtin_amdgcn_readlane(spos, s);
                    store_partial<D>(slab1 + ((int64_t)(r - 1) * SL + oldpos) * S::UNIT, blk[b], a.scale, lane);
                    const int64_t id = __builtin_amdgcn_readlane(nid, s);
                    blk[b].load(K1 + id * 16 * D * 2, V1 + id * 16 * D * 2, 16, bias2, lane);
                    blk[b].clear();
                }
            }
            sblk = keep ? sblk : nid;
            spos = keep ? npos : src;
        }
        __syncthreads();                                              // everyone is done with the previous rows
        stage_store<D, 64 * NW>(sr, qs, gs, st, tid);
        __syncthreads();
        for (int u = 0; u < 8; ++u) group_tile<D, NB>(qs, gs, st, u, o, blk, a.sc2, g);
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int pos = __builtin_amdgcn_readlane(spos, NB * wave + b);
        store_partial<D>(slab1 + ((int64_t)(a.GC - 1) * SL + pos) * S::UNIT, blk[b], a.scale, lane);
    }
}

// SS = sparse blocks a wave owns in one launch (blocks sparse_begin + wave, + 8, ...): a launch covers 8 SS of them;
// DENSE: may this instantiation take the shared dense block
template <int D, int SS, bool DENSE>
__global__ void __launch_bounds__(512) dkv_upper_kernel(LevelTable t, GroupArgs a) {
    using S = GShape<D>;
    __shared__ __attribute__((aligned(16))) char lds[2 * 256 * S::ROWB];   // Q rows | dO rows; the final reduction reuses it
    __shared__ __attribute__((aligned(16))) float st[512];
    char *qs = lds, *gs = lds + 256 * S::ROWB;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t per_head = a.NR / a.G;
    const int64_t grp = blockIdx.x;                                   // query group: G consecutive level-1 query blocks
    const int64_t bh = grp / per_head, R0 = (grp % per_head) * a.G;
    const TileOffsets<D> o = tile_offsets<D>(lane);

    const int nlev = min(t.nlev, a.lev_end);
    const int u_begin = t.bseg[2];                                    // first listed block of level 2
    const bool dense = DENSE && a.do_dense;
    BlockAcc<D> sp[SS][1], dn[DENSE ? 1 : 1];                         // this wave's sparse blocks; the dense block
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
        if (dense) {
            if ((a.nbs >> 6) != chunk) ctab.fill(t, bh, R0 * 16, u_begin, a.nbs >> 6, lane, D, nlev);
            dn[0].load(ctab.K(a.nbs & 63), ctab.V(a.nbs & 63), ctab.count(a.nbs & 63), ctab.bias(a.nbs & 63), lane);
        } else {
            dn[0].load(nullptr, nullptr, 16, 0.f, lane);
        }
        dn[0].clear();
    }

    StageRegs<D, 512> sr;
    stage_load<D, 512>(sr, a, bh * a.N + R0 * 256, tid);
    for (int r = 0; r < a.G; ++r) {
        stage_store<D, 512>(sr, qs, gs, st, tid);
        __syncthreads();
        if (r + 1 < a.G) stage_load<D, 512>(sr, a, bh * a.N + (R0 + r + 1) * 256, tid);   // flies during the math
#pragma unroll
        for (int s = 0; s < SS; ++s)
            if (a.sparse_begin + wave + 8 * s < a.nbs)
                for (int u = 0; u < 8; ++u) group_tile<D, 1>(qs, gs, st, u, o, sp[s], a.sc2, g);
        if (dense) group_tile<D, 1>(qs, gs, st, wave, o, dn, a.sc2, g);
        __syncthreads();                                              // everyone is done with this R's rows
    }

#pragma unroll
    for (int s = 0; s < SS; ++s) {
        const int jb = a.sparse_begin + wave + 8 * s;
        if (jb < a.nbs) store_partial<D>(partial_ptr<D>(t, a, nlev, u_begin + jb, grp), sp[s][0], a.scale, lane);
    }
    if constexpr (DENSE) {
        if (dense) {                                                  // the shared block: add the 8 waves' sums in wave order
            constexpr int SLOTS = 2 * S::NT;                          // f32x4 slots per wave: dK tiles, then dV tiles
            float *red = reinterpret_cast<float *>(lds);              // [wave][slot][lane] f32x4
            static_assert(8 * SLOTS * 64 * 16 <= 2 * 256 * S::ROWB, "the reduction must fit in the staged rows' memory");
#pragma unroll
            for (int n = 0; n < S::NT; ++n) {
                *reinterpret_cast<f32x4 *>(red + ((wave * SLOTS + n) * 64 + lane) * 4) = dn[0].accK[n];
                *reinterpret_cast<f32x4 *>(red + ((wave * SLOTS + S::NT + n) * 64 + lane) * 4) = dn[0].accV[n];
            }
            __syncthreads();
            float *dst = partial_ptr<D>(t, a, nlev, u_begin + a.nbs, grp) + i16 * D + 4 * g;
#pragma unroll
            for (int k = 0; k < SLOTS / 8; ++k) {                     // wave w owns slots w, w + 8, ...
                const int slot = wave + 8 * k;
                f32x4 sum = *reinterpret_cast<const f32x4 *>(red + (slot * 64 + lane) * 4);
#pragma unroll
                for (int w = 1; w < 8; ++w) {
                    const f32x4 x = *reinterpret_cast<const f32x4 *>(red + ((w * SLOTS + slot) * 64 + lane) * 4);
#pragma unroll
                    for (int c = 0; c < 4; ++c) sum[c] += x[c];
                }
                const bool isV = slot >= S::NT;
                const float w = __builtin_amdgcn_exp2f(dn[0].bias2) * (isV ? 1.f : a.scale);   // level weight (and scale for dK)
#pragma unroll
                for (int c = 0; c < 4; ++c) sum[c] *= w;
                *reinterpret_cast<f32x4 *>(dst + (isV ? 16 * D : 0) + (isV ? slot - S::NT : slot) * 16) = sum;
            }
        }
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
    const float *part;           // [bh][cnt][nblk][UNIT]
    const int32_t *C, *Iq, *I;   // key-major lists and I^(l) (null when dense)
    const float *upK, *upV;      // gradient of level l + 1 or null
    float *dstK, *dstV;          // [bh, n_l, D]
    int64_t cnt, n_l, nkb, rows; // listers per head, tokens, key blocks per head, rows of I^(l)
    int nblk, Kl, dense;
    int chain;                   // > 1: partials come from the chain kernel, which walked `chain` consecutive listers
};
template <int D, int NT>
__global__ void __launch_bounds__(NT) dkv_gather_kernel(GatherArgs a) {
    constexpr int U4 = GShape<D>::UNIT / 4, H4 = U4 / 2, PER = H4 / NT;   // float4 per partial / per half / per thread and half
    const int tid = threadIdx.x;
    const int64_t bh = blockIdx.x / a.nkb, j = blockIdx.x % a.nkb;
    const f32x4 *part = reinterpret_cast<const f32x4 *>(a.part);
    f32x4 k[PER], v[PER];
#pragma unroll
    for (int x = 0; x < PER; ++x) { k[x] = f32x4{0.f, 0.f, 0.f, 0.f}; v[x] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    if (a.dense) {
        const f32x4 *p = part + ((bh * a.cnt) * a.nblk + j) * U4;
#pragma unroll
        for (int x = 0; x < PER; ++x) { k[x] = p[tid + NT * x]; v[x] = p[H4 + tid + NT * x]; }
    } else {
        // first every thread resolves one lister (query block row and the position of j in that row's list),
        // NT at a time, then all threads add the partials in list order with independent loads
        __shared__ int64_t unit[NT];
        const int32_t beg = a.C[bh * (a.rows + 1) + j], end = a.C[bh * (a.rows + 1) + j + 1];
        const int32_t *lst = a.Iq + bh * a.rows * a.Kl;
        for (int32_t e0 = beg; e0 < end; e0 += NT) {
            const int32_t m = min(NT, end - e0);
            __syncthreads();
            if (tid < m) {
                const int64_t r = lst[e0 + tid];
                const int32_t *row = a.I + (bh * a.rows + r) * a.Kl;
                int pos = 0;
                for (int x = 0; x < a.Kl; ++x) pos += (row[x] < (int32_t)j) ? 1 : 0;   // rows are ascending
                int64_t un = ((bh * a.cnt + r) * a.nblk + pos) * U4;
                if (a.chain > 1 && r % a.chain != a.chain - 1) {                  // carried on by the next lister of the chain?
                    bool cont = false;
                    for (int x = 0; x < a.Kl; ++x) cont |= row[a.Kl + x] == (int32_t)j;
                    if (cont) un = -1;
                }
                unit[tid] = un;
            }
            __syncthreads();
#pragma unroll 4
            for (int32_t e = 0; e < m; ++e) {
                if (unit[e] < 0) continue;                                // same for every thread
                const f32x4 *p = part + unit[e];
#pragma unroll
                for (int x = 0; x < PER; ++x) { k[x] += p[tid + NT * x]; v[x] += p[H4 + tid + NT * x]; }
            }
        }
    }
#pragma unroll
    for (int x = 0; x < PER; ++x) {
        const int e4 = tid + NT * x;                                   // float4 index inside [16 keys][D channels]
        const int64_t tok = j * 16 + e4 / (D / 4);
        if (tok >= a.n_l) continue;
        const int col = (e4 % (D / 4)) * 4;
        f32x4 kk = k[x], vv = v[x];
        if (a.upK) {
            const int64_t up = (bh * ((a.n_l + 15) / 16) + j) * D + col;   // parent token of the block's 16 tokens
            kk += *reinterpret_cast<const f32x4 *>(a.upK + up) * 0.0625f;
            vv += *reinterpret_cast<const f32x4 *>(a.upV + up) * 0.0625f;
        }
        *reinterpret_cast<f32x4 *>(a.dstK + (bh * a.n_l + tok) * D + col) = kk;
        *reinterpret_cast<f32x4 *>(a.dstV + (bh * a.n_l + tok) * D + col) = vv;
    }
}

// Highest level the grouped kernels take; levels above it go to the split key-major kernel: a wide dense coarsest
// level (every query block would write a partial sum for every one of its key blocks, and summing over all queries
// is what the split kernel does in registers), and at d = 128 any dense level (no registers left for a shared block).
int dkv_group_top(const Plan &p) {
    if (p.Le == p.L && ((p.n[p.L] + 15) / 16 > 32 || p.d == 128)) return p.L - 1;
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

// Level-1 query blocks one workgroup of the chain kernel walks (1: the plain group kernel takes level 1).
// d = 64 with rows of 8 level-1 blocks, level 1 sparse and the only level the kernel is given.
// Measured at the headline: 8 query blocks per workgroup in 512 workgroups (two per CU) 259 us for the coarse stage,
// 4 in 1024: 275 us, 2: 297 us, 16 in 256 workgroups: 286 us, one query block per workgroup (no carrying): 357 us.
static int chain_len(const Plan &p) {
    if (p.d != 64 || p.L < 2 || p.Kl[1] != 8) return 1;
    if (upper_G(p) == 0 && dkv_group_top(p) > 1) return 1;
    const int64_t NR = p.N / 256;
    int GC = 8;
    while (GC > 1 && (NR % GC != 0 || (int64_t)p.bh * (NR / GC) < 512)) GC >>= 1;   // at least two workgroups per CU
    return GC;
}

// partial-slab layout: level 1 has one partial per (level-1 query block, list position), levels >= 2 one per
// (query group, list position)
static int64_t slab_layout(const Plan &p, int64_t *lvl_off, int *nblk, int64_t *groups) {
    const int64_t NR = p.N / 256, unit = 2 * 16 * p.d;
    const int G = upper_G(p);
    int64_t off = 0;
    for (int l = 0; l <= kMaxL; ++l) { lvl_off[l] = 0; nblk[l] = 0; groups[l] = 0; }
    for (int l = 1; l <= dkv_group_top(p); ++l) {
        nblk[l] = l < p.L ? p.Kl[l] : (int)((p.n[l] + 15) / 16);
        groups[l] = (l >= 2 && G) ? NR / G : NR;
        lvl_off[l] = off;
        off += (int64_t)p.bh * groups[l] * nblk[l] * unit;
    }
    return off;
}

// bytes of the partial slab and of each of the two reduction buffers
void dkv_group_sizes(const Plan &p, size_t *slab_bytes, size_t *red_bytes) {
    const int64_t NR = p.N / 256, unit = 2 * 16 * p.d;
    int64_t lvl_off[kMaxL + 1], groups[kMaxL + 1];
    int nblk[kMaxL + 1];
    *slab_bytes = (size_t)slab_layout(p, lvl_off, nblk, groups) * sizeof(float);
    size_t red = 0;
    for (int l = 1; l <= dkv_group_top(p); ++l) {
        const size_t r = (size_t)p.bh * ((NR + 15) / 16) * nblk[l] * unit * sizeof(float);
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
    const int64_t unit = 2 * 16 * p.d;
    const bool dense = (l == p.L);
    const float *cur = a.slab + a.lvl_off[l];
    int64_t cnt = groups;
    const int64_t target = dense ? 1 : p.n[l + 1];          // listers per head: level-l query blocks, or the head
    const int64_t width4 = (int64_t)a.nblk[l] * (unit / 4);
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
    ga.chain = l == 1 ? a.GC : 1;
    const dim3 grid((unsigned)(p.bh * ga.nkb));
    // latency-bound (lists -> rows of I -> partials): more, smaller workgroups per CU shorten the launch
    if (p.d == 64) dkv_gather_kernel<64, 128><<<grid, 128, 0, s>>>(ga);
    else dkv_gather_kernel<128, 256><<<grid, 256, 0, s>>>(ga);
    return hipGetLastError();
}

static hipError_t launch_group_kernel(const Plan &p, const LevelTable &t, const GroupArgs &a, hipStream_t s) {
    if (a.GC > 1) {
        dkv_chain_kernel<64, 4, 2><<<dim3((unsigned)(p.bh * (a.NR / a.GC))), 256, 0, s>>>(t, a);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)(p.bh * a.NR));
    if (p.d == 64) dkv_group_kernel<64, 4, 2><<<grid, 256, 0, s>>>(t, a);
    else dkv_group_kernel<128, 8, 1><<<grid, 512, 0, s>>>(t, a);
    return hipGetLastError();
}

hipError_t launch_dkv_group(const Plan &p, const LevelTable &t, const void *Q, const void *dO, const float *LSE,
                            const float *D, void *ws, hipStream_t s, hipEvent_t lists, hipStream_t side,
                            hipEvent_t upper_done) {
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
    a.GC = chain_len(p);
    upper_blocks(p, &a.nbs, &a.nbd);
    a.sparse_begin = 0;
    a.do_dense = 0;

    // first the kernels that write the partials (they read no list), then, top-down, the reductions and gathers
    // (a level adds the share of the one above)
    if (G) {                                                // levels >= 2 in their own kernel
        GroupArgs up = a;
        up.lev_end = top + 1;
        const dim3 grid((unsigned)(p.bh * (NR / G)));
        const int per_launch = p.d == 64 ? 16 : 8;          // sparse blocks one launch covers
        for (int sb = 0; sb == 0 || sb < up.nbs; sb += per_launch) {   // the first launch also takes the dense block (d = 64)
            up.sparse_begin = sb;
            up.do_dense = (sb == 0 && up.nbd > 0) ? 1 : 0;
            if (p.d == 128) dkv_upper_kernel<128, 1, false><<<grid, 512, 0, s>>>(t, up);
            else if (up.nbs - sb > 8) dkv_upper_kernel<64, 2, true><<<grid, 512, 0, s>>>(t, up);
            else dkv_upper_kernel<64, 1, true><<<grid, 512, 0, s>>>(t, up);
            GRP_TRY(hipGetLastError());
        }
    }
    // With a side stream (the one the lists are made on), the small reductions and gathers of levels >= 2 follow the
    // lists there, beside the level-1 kernel, and `lists` is recorded again behind them.
    const bool split = G && side && lists && upper_done && top >= 2;
    if (split) {
        GRP_TRY(hipEventRecord(upper_done, s));
        GRP_TRY(hipStreamWaitEvent(side, upper_done, 0));
        for (int l = top; l >= 2; --l) GRP_TRY(finish_level(p, t, a, l, groups[l], w, side));
        GRP_TRY(hipEventRecord(lists, side));
    }
    a.lev_end = G ? 2 : top + 1;
    GRP_TRY(launch_group_kernel(p, t, a, s));
    if (lists) GRP_TRY(hipStreamWaitEvent(s, lists, 0));
    for (int l = split ? 1 : top; l >= 1; --l) GRP_TRY(finish_level(p, t, a, l, groups[l], w, s));
    return hipSuccess;
}

}  // namespace llsa
