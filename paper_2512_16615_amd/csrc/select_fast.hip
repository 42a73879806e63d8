// Hierarchical Top-K selection, one level (Alg. 1, selection loop), fast path for bf16, B in {16, 32, 64} and
// K <= 64: at most 256 candidates per query tile (select_fast_kernel) or any number (select_dense_kernel).
//
// One workgroup (256 threads) per level-l query block of 16 query tokens.  The candidate key rows (all
// n_L tokens at the coarsest level, the 16 * K_l children of the parent's picks below it) and the 16
// query rows are staged once in LDS; lane (row r, column group c) scores candidates c, c + 16, ... of
// row r, so all scores of a row sit in one 16-lane row group and the Top-K runs in registers.
// Scores are fp32 fused-multiply-add chains over channels 0 .. d-1 in order (the same chain on every
// launch shape), ties go to the lower key id, rows are written in ascending id order.
#include "mfma_common.h"

namespace llsa {

__device__ __forceinline__ void unpack8(u32x4 w, float *f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// The coarsest level's selection for kernels that run the level below it in the same launch (TOP).
struct TopLevel {
    const uint16_t *Q, *K;       // Q^(L), K^(L): [bh, n, D]
    int32_t *out;                // I^(L-1): [bh, n, Kp]
    int n;                       // tokens of level L per head (<= 64)
};

// MC = candidates per lane (8: up to 128 candidates, 16: up to 256); KW = winners per lane (K <= 16 KW).
// TOP: this launch is level L-1 and also does level L (Alg. 1's first selection step, dense over the n_L <= 64
// coarsest tokens): every workgroup scores the level-L token above its 16 queries against all level-L keys on its
// first wave (same fp32 multiply-add chain, same tie rule), which gives the row of I^(L-1) it needs as `parent`; the
// workgroup at the start of that row's B queries also writes it out.  One launch less on a latency-bound path.
template <int D, int MC, int KW, bool TOP>
__global__ void __launch_bounds__(256) select_fast_kernel(const uint16_t *__restrict__ Ql, const uint16_t *__restrict__ Kl,
                                                           int64_t n_l, const int32_t *__restrict__ parent, int Kp,
                                                           int Kout, int32_t *__restrict__ out, int C, int64_t nblk,
                                                           int lb, TopLevel top) {
    constexpr int STRIDE = 2 * D + 16;                      // bytes per staged row: keeps 16-byte reads conflict-free
    constexpr int CH = D / 8;                               // 16-byte chunks per row
    __shared__ __attribute__((aligned(16))) char kc[16 * MC * STRIDE];
    __shared__ __attribute__((aligned(16))) char qs[16 * STRIDE];

    const int tid = threadIdx.x;
    const int64_t bh = blockIdx.x / nblk, r = blockIdx.x % nblk;
    const uint16_t *Kb = Kl + bh * n_l * D;
    // the 16 query tokens lie in one block of B = 2^lb tokens: row (16 r) / B of the parent list, whose picks'
    // B children each are the candidates
    const int Bm1 = (1 << lb) - 1;
    const int32_t *prow = parent ? parent + (bh * (n_l >> lb) + (r >> (lb - 4))) * Kp : nullptr;
    if constexpr (TOP) {
        __shared__ int32_t prow_sh[16];
        if (tid < 64) {
            const int64_t q = r >> (lb - 4);                 // the level-L token above this query block
            float sc = -INFINITY;
            if (tid < top.n) {
                const uint16_t *qrow = top.Q + (bh * top.n + q) * D, *krow = top.K + (bh * top.n + tid) * D;
                sc = 0.f;
                for (int ch = 0; ch < CH; ++ch) {
                    float qf[8], kf[8];
                    unpack8(*reinterpret_cast<const u32x4 *>(qrow + ch * 8), qf);
                    unpack8(*reinterpret_cast<const u32x4 *>(krow + ch * 8), kf);
#pragma unroll
                    for (int e = 0; e < 8; ++e) sc = __builtin_fmaf(qf[e], kf[e], sc);
                }
            }
            int won = 0x7fffffff;                            // lane k: the k-th winner's key id
            for (int k = 0; k < Kp; ++k) {
                float bs = sc;
                int bp = tid;
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) {
                    const float os = __shfl_xor(bs, o, 64);
                    const int op = __shfl_xor(bp, o, 64);
                    if (os > bs || (os == bs && op < bp)) { bs = os; bp = op; }
                }
                if (bp == tid) sc = -INFINITY;
                if (tid == k) won = bp;
            }
            int rank = 0;                                    // rows are stored in ascending id order
            for (int k = 0; k < Kp; ++k) rank += (__shfl(won, k, 64) < won) ? 1 : 0;
            if (tid < Kp) {
                prow_sh[rank] = won;
                if ((r & ((1 << (lb - 4)) - 1)) == 0) top.out[(bh * top.n + q) * Kp + rank] = won;
            }
        }
        __syncthreads();
        prow = prow_sh;
    }

    // stage the candidate rows (16-byte chunks, coalesced within a row) and the query rows
    for (int c = tid; c < C * CH; c += 256) {
        const int p = c / CH, part = c % CH;
        const int64_t id = prow ? ((int64_t)prow[p >> lb] << lb) + (p & Bm1) : p;
        *reinterpret_cast<u32x4 *>(kc + p * STRIDE + part * 16) = *reinterpret_cast<const u32x4 *>(Kb + id * D + part * 8);
    }
    for (int c = tid; c < 16 * CH; c += 256) {
        const int u = c / CH, part = c % CH;
        const int64_t i = min(r * 16 + u, n_l - 1);          // rows past a ragged end are computed but not stored
        *reinterpret_cast<u32x4 *>(qs + u * STRIDE + part * 16) =
            *reinterpret_cast<const u32x4 *>(Ql + (bh * n_l + i) * D + part * 8);
    }
    __syncthreads();

    const int cg = tid & 15, row = tid >> 4;                // 16 consecutive lanes share a query row
    float sc[MC];
#pragma unroll
    for (int m = 0; m < MC; ++m) sc[m] = 0.f;
    for (int ch = 0; ch < CH; ++ch) {
        float q[8];
        unpack8(*reinterpret_cast<const u32x4 *>(qs + row * STRIDE + ch * 16), q);
#pragma unroll
        for (int m = 0; m < MC; ++m) {
            const int p = min(cg + 16 * m, C - 1);
            float k[8];
            unpack8(*reinterpret_cast<const u32x4 *>(kc + p * STRIDE + ch * 16), k);
#pragma unroll
            for (int e = 0; e < 8; ++e) sc[m] = __builtin_fmaf(q[e], k[e], sc[m]);
        }
    }
#pragma unroll
    for (int m = 0; m < MC; ++m)
        if (cg + 16 * m >= C) sc[m] = -INFINITY;

    // K rounds of arg-max over the row's candidates (score descending, position ascending)
    int mine[KW];                                           // lane k % 16 of the row group keeps the k-th winner
#pragma unroll
    for (int w = 0; w < KW; ++w) mine[w] = 0;
    for (int k = 0; k < Kout; ++k) {
        float bs = sc[0];
        int bp = cg;
#pragma unroll
        for (int m = 1; m < MC; ++m)
            if (sc[m] > bs) { bs = sc[m]; bp = cg + 16 * m; }   // ascending positions: strict '>' keeps the lowest
#pragma unroll
        for (int o = 8; o >= 1; o >>= 1) {
            const float os = __shfl_xor(bs, o, 16);
            const int op = __shfl_xor(bp, o, 16);
            if (os > bs || (os == bs && op < bp)) { bs = os; bp = op; }
        }
#pragma unroll
        for (int m = 0; m < MC; ++m)
            if (bp == cg + 16 * m) sc[m] = -INFINITY;
#pragma unroll
        for (int w = 0; w < KW; ++w)
            if (k == cg + 16 * w) mine[w] = bp;
    }
    // candidate positions ascend with key id (parent rows are ascending): rank the winners by position
    int rank[KW];
#pragma unroll
    for (int w = 0; w < KW; ++w) rank[w] = 0;
#pragma unroll
    for (int w2 = 0; w2 < KW; ++w2)
        for (int k = 0; k < 16 && 16 * w2 + k < Kout; ++k) {
            const int other = __shfl(mine[w2], k, 16);
#pragma unroll
            for (int w = 0; w < KW; ++w) rank[w] += (other < mine[w]) ? 1 : 0;
        }
    const int64_t i = r * 16 + row;
#pragma unroll
    for (int w = 0; w < KW; ++w)
        if (cg + 16 * w < Kout && i < n_l) {
            const int64_t id = prow ? ((int64_t)prow[mine[w] >> lb] << lb) + (mine[w] & Bm1) : mine[w];
            out[(bh * n_l + i) * Kout + rank[w]] = (int32_t)id;
        }
}

// More than 256 candidates: a coarsest level of more than 256 tokens (few levels for the sequence length, or the
// single-level method of Sec. 3.2: every token of the level is a candidate), or more than 256 children of the parent's
// picks (B = 64, K > 4).  Same lane layout; the C candidates pass through LDS 256 at a time, and the row group
// keeps its K best so far (lane k: the k-th best), which compete in the next chunk's rounds as one more candidate
// per lane.  Their key ids are lower than the chunk's (candidate positions ascend with the key id), so the tie
// rule holds.
template <int D, int KW>
__global__ void __launch_bounds__(256) select_dense_kernel(const uint16_t *__restrict__ Ql, const uint16_t *__restrict__ Kl,
                                                            int64_t n_l, const int32_t *__restrict__ parent, int Kp, int C,
                                                            int Kout, int32_t *__restrict__ out, int64_t nblk, int lb) {
    constexpr int STRIDE = 2 * D + 16, CH = D / 8, MC = 16;
    __shared__ __attribute__((aligned(16))) char kc[256 * STRIDE];
    __shared__ __attribute__((aligned(16))) char qs[16 * STRIDE];

    const int tid = threadIdx.x;
    const int64_t bh = blockIdx.x / nblk, r = blockIdx.x % nblk;
    const uint16_t *Kb = Kl + bh * n_l * D;
    const int Bm1 = (1 << lb) - 1;
    const int32_t *prow = parent ? parent + (bh * (n_l >> lb) + (r >> (lb - 4))) * Kp : nullptr;
    auto key_id = [&](int pos) { return prow ? (prow[pos >> lb] << lb) + (pos & Bm1) : pos; };
    for (int c = tid; c < 16 * CH; c += 256) {
        const int u = c / CH, part = c % CH;
        const int64_t i = min(r * 16 + u, n_l - 1);
        *reinterpret_cast<u32x4 *>(qs + u * STRIDE + part * 16) =
            *reinterpret_cast<const u32x4 *>(Ql + (bh * n_l + i) * D + part * 8);
    }
    const int cg = tid & 15, row = tid >> 4;
    constexpr int kNone = 0x7fffffff;
    float best_s[KW];                                       // lane k % 16 of the row group: k-th best so far and its key id
    int best_id[KW];
#pragma unroll
    for (int w = 0; w < KW; ++w) { best_s[w] = -INFINITY; best_id[w] = kNone; }
    for (int c0 = 0; c0 < C; c0 += 256) {
        __syncthreads();                                    // the previous chunk has been scored
        for (int c = tid; c < 256 * CH; c += 256) {
            const int p = c / CH, part = c % CH;
            const int64_t id = key_id(min(c0 + p, C - 1));
            *reinterpret_cast<u32x4 *>(kc + p * STRIDE + part * 16) = *reinterpret_cast<const u32x4 *>(Kb + id * D + part * 8);
        }
        __syncthreads();
        float sc[MC];
#pragma unroll
        for (int m = 0; m < MC; ++m) sc[m] = 0.f;
        for (int ch = 0; ch < CH; ++ch) {
            float q[8];
            unpack8(*reinterpret_cast<const u32x4 *>(qs + row * STRIDE + ch * 16), q);
#pragma unroll
            for (int m = 0; m < MC; ++m) {
                float k[8];
                unpack8(*reinterpret_cast<const u32x4 *>(kc + (cg + 16 * m) * STRIDE + ch * 16), k);
#pragma unroll
                for (int e = 0; e < 8; ++e) sc[m] = __builtin_fmaf(q[e], k[e], sc[m]);
            }
        }
        const int pos0 = c0 + cg;                           // candidate position of sc[m]: pos0 + 16 m
        int id[MC];                                         // and its key id (ascending with the position)
#pragma unroll
        for (int m = 0; m < MC; ++m) {
            id[m] = pos0 + 16 * m < C ? key_id(pos0 + 16 * m) : kNone;
            if (pos0 + 16 * m >= C) sc[m] = -INFINITY;
        }

        float old_s[KW], new_s[KW];                         // this lane's entries of the running list compete too
        int old_id[KW], new_id[KW];
#pragma unroll
        for (int w = 0; w < KW; ++w) { old_s[w] = best_s[w]; old_id[w] = best_id[w]; new_s[w] = -INFINITY; new_id[w] = kNone; }
        for (int k = 0; k < Kout; ++k) {
            float bs = old_s[0];
            int bp = old_id[0];
#pragma unroll
            for (int w = 1; w < KW; ++w)                          // the running entries are in no id order
                if (old_s[w] > bs || (old_s[w] == bs && old_id[w] < bp)) { bs = old_s[w]; bp = old_id[w]; }
#pragma unroll
            for (int m = 0; m < MC; ++m)
                if (sc[m] > bs) { bs = sc[m]; bp = id[m]; }      // ids above the running ones, ascending: strict '>'
#pragma unroll
            for (int o = 8; o >= 1; o >>= 1) {
                const float os = __shfl_xor(bs, o, 16);
                const int op = __shfl_xor(bp, o, 16);
                if (os > bs || (os == bs && op < bp)) { bs = os; bp = op; }
            }
#pragma unroll
            for (int w = 0; w < KW; ++w)
                if (bp == old_id[w]) { old_s[w] = -INFINITY; old_id[w] = kNone; }
#pragma unroll
            for (int m = 0; m < MC; ++m)
                if (bp == id[m]) sc[m] = -INFINITY;
#pragma unroll
            for (int w = 0; w < KW; ++w)
                if (k == cg + 16 * w) { new_s[w] = bs; new_id[w] = bp; }
        }
#pragma unroll
        for (int w = 0; w < KW; ++w) { best_s[w] = new_s[w]; best_id[w] = new_id[w]; }
    }
    int rank[KW];                                           // rows are written in ascending id order
#pragma unroll
    for (int w = 0; w < KW; ++w) rank[w] = 0;
#pragma unroll
    for (int w2 = 0; w2 < KW; ++w2)
        for (int k = 0; k < 16 && 16 * w2 + k < Kout; ++k) {
            const int other = __shfl(best_id[w2], k, 16);
#pragma unroll
            for (int w = 0; w < KW; ++w) rank[w] += (other < best_id[w]) ? 1 : 0;
        }
    const int64_t i = r * 16 + row;
#pragma unroll
    for (int w = 0; w < KW; ++w)
        if (cg + 16 * w < Kout && i < n_l) out[(bh * n_l + i) * Kout + rank[w]] = best_id[w];
}

// true if the fast kernel covers this level
bool select_fast_ok(const Plan &p, int l) {
    const int64_t C = (l == p.L) ? p.n[l] : (int64_t)p.Kl[l] * p.B;
    // any number of candidates (256 at a time beyond 256); 16 consecutive query tokens share their candidates
    return p.fast && p.Kl[l - 1] <= 64 && p.n[l] < ((int64_t)1 << 30) && C < (1 << 30) &&
           (l == p.L || p.n[l] % 16 == 0);
}

// Can level L be done inside level L-1's launch?
bool select_top_fused(const Plan &p) {
    if (p.L < 2 || p.desc.kernel_path != 0 || !select_fast_ok(p, p.L) || !select_fast_ok(p, p.L - 1)) return false;
    return p.n[p.L] <= 64 && p.Kl[p.L - 1] <= 16 && p.Kl[p.L - 1] * p.B <= 256;
}

hipError_t launch_select_fast(const Plan &p, int l, const void *ws, const int32_t *parent, int32_t *out, hipStream_t s,
                              int32_t *top_out) {
    const char *w = static_cast<const char *>(ws);
    const bool top = (l == p.L);
    const int64_t nblk = (p.n[l] + 15) / 16;
    const uint16_t *Ql = (const uint16_t *)(w + p.pyr_off[0][l]), *Kl = (const uint16_t *)(w + p.pyr_off[1][l]);
    const int32_t *par = top ? nullptr : parent;
    const int Kp = top ? 0 : p.Kl[l], Kout = p.Kl[l - 1];
    dim3 grid((unsigned)(p.bh * nblk));
    const int C = top ? (int)p.n[l] : p.Kl[l] * p.B;
    const bool wide = Kout > 16;                            // up to 4 winners per lane instead of one
    TopLevel tl = {nullptr, nullptr, nullptr, 0};
#define LLSA_SEL(kernel, ...) kernel<<<grid, 256, 0, s>>>(__VA_ARGS__)
    if (top_out) {                                          // level L-1 with level L inside (select_top_fused)
        tl.Q = (const uint16_t *)(w + p.pyr_off[0][p.L]);
        tl.K = (const uint16_t *)(w + p.pyr_off[1][p.L]);
        tl.out = top_out;
        tl.n = (int)p.n[p.L];
        if (p.d == 64) {
            if (C <= 128 && !wide) LLSA_SEL((select_fast_kernel<64, 8, 1, true>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
            else if (!wide) LLSA_SEL((select_fast_kernel<64, 16, 1, true>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
            else LLSA_SEL((select_fast_kernel<64, 16, 4, true>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
        } else {
            if (C <= 128 && !wide) LLSA_SEL((select_fast_kernel<128, 8, 1, true>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
            else if (!wide) LLSA_SEL((select_fast_kernel<128, 16, 1, true>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
            else LLSA_SEL((select_fast_kernel<128, 16, 4, true>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
        }
        return hipGetLastError();
    }
    if (C > 256) {
        if (p.d == 64 && !wide) LLSA_SEL((select_dense_kernel<64, 1>), Ql, Kl, p.n[l], par, Kp, C, Kout, out, nblk, p.lb);
        else if (p.d == 64) LLSA_SEL((select_dense_kernel<64, 4>), Ql, Kl, p.n[l], par, Kp, C, Kout, out, nblk, p.lb);
        else if (!wide) LLSA_SEL((select_dense_kernel<128, 1>), Ql, Kl, p.n[l], par, Kp, C, Kout, out, nblk, p.lb);
        else LLSA_SEL((select_dense_kernel<128, 4>), Ql, Kl, p.n[l], par, Kp, C, Kout, out, nblk, p.lb);
        return hipGetLastError();
    }
    if (p.d == 64) {
        if (C <= 128 && !wide) LLSA_SEL((select_fast_kernel<64, 8, 1, false>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
        else if (!wide) LLSA_SEL((select_fast_kernel<64, 16, 1, false>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
        else LLSA_SEL((select_fast_kernel<64, 16, 4, false>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
    } else {
        if (C <= 128 && !wide) LLSA_SEL((select_fast_kernel<128, 8, 1, false>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
        else if (!wide) LLSA_SEL((select_fast_kernel<128, 16, 1, false>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
        else LLSA_SEL((select_fast_kernel<128, 16, 4, false>), Ql, Kl, p.n[l], par, Kp, Kout, out, C, nblk, p.lb, tl);
    }
#undef LLSA_SEL
    return hipGetLastError();
}

}  // namespace llsa
