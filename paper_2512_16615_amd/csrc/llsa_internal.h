// Internal declarations shared by the translation units of libllsa (host plan + kernel launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/llsa.h"

namespace llsa {

constexpr int kMaxL = 8;            // coarse levels supported (levels 0..8)
constexpr int kMaxCand = 4096;      // candidates per selection row held in LDS (n_L or K_l * B)

// Host-side description of one problem: level table and buffer layout.
struct Plan {
    llsa_desc desc;
    int L, Le, B, K, d, bh, elt;    // elt = bytes per element of the I/O type
    int64_t N;
    float scale;
    int64_t n[kMaxL + 1];           // tokens per head at level l
    int Kl[kMaxL];                  // K_l = min(K, n_{l+1})
    size_t idx_off[kMaxL];          // byte offset of I^(l) inside `indices`
    size_t idx_bytes;
    size_t pyr_off[3][kMaxL + 1];   // workspace byte offset of pooled level l (1..L) of Q/K/V
    size_t D_off;                   // [bh, N] fp32: rowsum(dO * O)
    size_t C_off[kMaxL], cnt_off[kMaxL], Iq_off[kMaxL], Iqtmp_off[kMaxL];
    size_t dKacc_off[kMaxL + 1], dVacc_off[kMaxL + 1]; // fp32 gradients of pooled level l (1..L)
    size_t part_off, part_bytes;    // partial sums of split key-major reductions
    size_t grp_slab_off, grp_red_off[2];   // partials of the query-grouped coarse dK/dV kernel and its reductions
    bool group;                     // coarse levels' dK/dV run grouped by level-1 query block
    size_t ws_fwd, ws_bwd;
    int list_len;                   // tokens one query attends to
    bool fast;                      // MFMA kernels apply (bf16, B in {16, 32, 64}, d in {64, 128})
    int lb;                         // log2 B when fast
};

// What the attention-type kernels need to walk the gathered list of a query block.
struct LevelTable {
    const void *K[kMaxL + 1];       // level-l keys   [bh, n_l, d]
    const void *V[kMaxL + 1];       // level-l values [bh, n_l, d]
    const int32_t *I[kMaxL + 1];    // I^(l) [bh, rows_l, K_l]; unused for l = L
    int64_t n[kMaxL + 1];
    int64_t rows[kMaxL + 1];
    int64_t Bpow[kMaxL + 2];        // B^l
    int Kl[kMaxL + 1];
    int seg[kMaxL + 2];             // list position where level l starts; seg[nlev] = list length
    int bseg[kMaxL + 2];            // same in units of 16-token key blocks (used when B = 16)
    float bias[kMaxL + 1];          // l * ln B (or 0)
    int nlev;                       // levels in the list = Le + 1
    int L, B, d;
    int lb, ls;                     // log2 B and log2(B / 16) when B is 16, 32 or 64 (MFMA kernels), else 0
    float scale;
};

LevelTable make_level_table(const Plan &p, const void *K0, const void *V0, const int32_t *indices,
                            const void *workspace);

// ---- portable scalar kernels (any supported shape) ----
hipError_t launch_pool(const Plan &p, const void *Q, const void *K, const void *V, void *ws, bool q_too,
                       hipStream_t s);
// QK-Norm + RoPE of Q and K fused with level-1 pooling, then the remaining pooled levels (fills Qout, Kout and ws)
hipError_t launch_qknorm_rope_pool(const Plan &p, const void *Qpre, const void *Kpre, const void *V,
                                   const float *gamma_q, const float *gamma_k, const float *cos_t, const float *sin_t,
                                   float eps, void *Qout, void *Kout, void *ws, hipStream_t s);
hipError_t launch_select(const Plan &p, int l, const void *ws, const int32_t *parent, int32_t *out, hipStream_t s);
hipError_t launch_attn_fwd_generic(const Plan &p, const LevelTable &t, const void *Q, void *O, float *LSE,
                                   hipStream_t s);
hipError_t launch_bwd_pre(const Plan &p, const void *O, const void *dO, float *D, hipStream_t s);
hipError_t launch_csc(const Plan &p, int top_level, const int32_t *I, void *ws, hipStream_t s);  // levels 0..top_level
// level 0's key-major lists through a dense T x T block mask (`mask`: bh * T * T bytes, rounded up to 16) instead of Alg. 2
hipError_t launch_mask_lists(const Plan &p, const int32_t *indices, void *ws, void *mask, hipStream_t s);
hipError_t launch_dq_generic(const Plan &p, const LevelTable &t, const void *Q, const void *dO, const float *LSE,
                             const float *D, void *dQ, hipStream_t s);
hipError_t launch_dkv_generic(const Plan &p, const LevelTable &t, int l, const void *Q, const void *dO,
                              const float *LSE, const float *D, void *ws, void *dK, void *dV, hipStream_t s);
hipError_t launch_unpool(const Plan &p, int l, void *ws, hipStream_t s);
// nested-patch token order of a 2^bits x 2^bits grid (or back); rows of row_bytes (a multiple of 16) bytes
hipError_t launch_reorder(int64_t bh, int64_t N, int row_bytes, int bits, int inverse, const void *in, void *out,
                          hipStream_t s);

// ---- fast selection (bf16, B = 16 / 32 / 64, K <= 64; any number of candidates, 256 at a time) ----
bool select_fast_ok(const Plan &p, int l);
// top_out != null: l = L - 1 and the launch also does level L, writing I^(L-1) to top_out (allowed if select_top_fused)
hipError_t launch_select_fast(const Plan &p, int l, const void *ws, const int32_t *parent, int32_t *out, hipStream_t s,
                              int32_t *top_out = nullptr);
bool select_top_fused(const Plan &p);

// ---- bf16 MFMA kernels (B = 16 / 32 / 64, d = 64 or 128, N % 64 == 0) ----
hipError_t launch_attn_fwd_mfma(const Plan &p, const LevelTable &t, const void *Q, void *O, float *LSE, hipStream_t s);
// variant that shares the coarse levels among the 8 or 16 sibling query blocks of a workgroup (N % 256 == 0)
hipError_t launch_attn_fwd_shared(const Plan &p, const LevelTable &t, const void *Q, void *O, float *LSE,
                                  hipStream_t s);
// also writes D = rowsum(dO * O) for the key-major kernels that follow
hipError_t launch_dq_mfma(const Plan &p, const LevelTable &t, const void *Q, const void *O, const void *dO,
                          const float *LSE, float *D, void *dQ, hipStream_t s);
hipError_t launch_dq_shared(const Plan &p, const LevelTable &t, const void *Q, const void *O, const void *dO,
                            const float *LSE, float *D, void *dQ, hipStream_t s);
// key-major dK/dV of level l; levels >= 1 also fold their split slabs and the level above into the
// level's fp32 gradient buffer, so they must be launched from the coarsest level down
hipError_t launch_dkv_mfma(const Plan &p, const LevelTable &t, int l, const void *Q, const void *dO, const float *LSE,
                           const float *D, void *ws, void *dK, void *dV, hipStream_t s, bool level0_alone = false);
int dkv_splits(const Plan &p, int l);    // workgroups sharing one key block's query list at level l
// all coarse levels (dkv_group_top .. 1) at once, grouped by level-1 query block; fills the levels' fp32
// gradients.  `lists` (or null): event after which the key-major lists are complete, recorded on another stream;
// `s` waits for it behind the kernels that need no list, before the gathers.  `side`, `upper_done` (or null): the
// stream the lists are made on and a spare event; the reductions and gathers of levels >= 2 then run on `side` behind
// the lists, beside the level-1 kernel, and `lists` is recorded once more behind them (so it still marks the end of `side`).
hipError_t launch_dkv_group(const Plan &p, const LevelTable &t, const void *Q, const void *dO, const float *LSE,
                            const float *D, void *ws, hipStream_t s, hipEvent_t lists, hipStream_t side = nullptr,
                            hipEvent_t upper_done = nullptr);
void dkv_group_sizes(const Plan &p, size_t *slab_bytes, size_t *red_bytes);
int dkv_group_top(const Plan &p);         // highest level the grouped kernel takes (the rest: split kernel)

// ---- measured peaks for the benchmark (calibrate.hip) ----
hipError_t launch_peak_mfma(float *out, int iters, int workgroups, hipStream_t s);
hipError_t launch_peak_copy(const void *src, void *dst, int64_t bytes, hipStream_t s);

}  // namespace llsa
