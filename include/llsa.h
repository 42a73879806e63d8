/*
 * llsa.h - C ABI of the MI355X (gfx950) Log-linear Sparse Attention library.
 *
 * One attention layer, forward and backward, as defined by Alg. 1 of the paper
 * ("Log-linear Sparse Attention"): hierarchical compression, hierarchical
 * Top-K selection, attention with Hierarchical KV Enrichment and KV
 * Reweighting; backward through the selection lists (Sec. 4.3, Alg. 2).
 *
 * Conventions for every entry point
 *   - Pointers named Q, K, V, O, dO, dQ, dK, dV, LSE, indices, workspace and
 *     every pointer of the step-wise calls are DEVICE pointers owned by the
 *     caller; `const llsa_desc*`, the plan and all `out` pointers of the query
 *     functions are HOST pointers.
 *   - Tensors are [batch, heads, N, d], contiguous, d innermost, element type
 *     `desc.dtype` (fp32, or bf16 stored as 16-bit words).
 *   - The library allocates no device memory, never synchronises the host and
 *     only enqueues work on the given HIP stream (`hip_stream` is a
 *     hipStream_t passed as void*; NULL = the default stream).
 *   - All validation happens on the host before anything is enqueued: on any
 *     status other than LLSA_OK no kernel has been launched and no output has
 *     been touched (LLSA_ERR_RUNTIME excepted: a launch itself failed).
 *   - Indices are 0-based.  Level l has n_l = N / B^l tokens (l = 0..L);
 *     I^(l) (l = 0..L-1) has n_{l+1} rows of K_l = min(K, n_{l+1}) key-block
 *     ids at level l, each row sorted ascending.
 */
#ifndef LLSA_H
#define LLSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LLSA_OK = 0,
    LLSA_ERR_NULL = 1,        /* a required pointer is NULL                              */
    LLSA_ERR_BAD_SHAPE = 2,   /* N not divisible by B^L, L < 1, Le outside 0..L, K < 1...; a tensor, LSE or
                                 indices pointer not 16-byte aligned, a workspace not 256-byte aligned */
    LLSA_ERR_UNSUPPORTED = 3, /* a (d, B, K, dtype, size) combination no kernel handles  */
    LLSA_ERR_WORKSPACE = 4,   /* llsa_forward_static: the plan needs more than the static workspace */
    LLSA_ERR_RUNTIME = 5      /* a HIP launch failed                                     */
} llsa_status;

typedef enum { LLSA_F32 = 0, LLSA_BF16 = 1 } llsa_dtype;

/* Problem statement of Alg. 1 (its Input line) plus the knobs the paper leaves open. */
typedef struct {
    int32_t batch, heads;
    int64_t N;          /* tokens per head; must be divisible by B^L                       */
    int32_t d;          /* head dimension: 16, 32, 64 or 128                                */
    int32_t B;          /* block size (2..64)                                               */
    int32_t K;          /* Top-K parameter, same at every level (Sec. 4.1)                  */
    int32_t L;          /* number of coarse levels (>= 1)                                   */
    int32_t Le;         /* KV-enrichment levels, 0..L; Le = L is the paper's default        */
    float sm_scale;     /* logits = sm_scale * q.k (+ l ln B); <= 0 selects 1/sqrt(d)       */
    int32_t dtype;      /* llsa_dtype of Q, K, V, O and the gradients                       */
    int32_t reweight;   /* 1: a level-l token weighs B^l (KV Reweighting); 0: weight 1      */
    int32_t bwd_repool; /* 1: llsa_backward rebuilds the pooled K/V levels from K, V, so the
                           workspace need not survive between the two calls; 0: backward is
                           given the very workspace llsa_forward filled                     */
    int32_t kernel_path;/* 0: fastest kernels available for the shape; 1: force the portable
                           scalar kernels (any supported shape, used as a cross-check)      */
    int32_t single_stream; /* 0: llsa_backward may run the index transpose, which depends on
                           the indices only, on one auxiliary stream the plan owns, beside
                           kernels that do not read its lists; the stream is forked from
                           and joined back into the caller's stream inside the call, so
                           the caller sees plain stream order; 1: everything goes to the
                           caller's stream                                                  */
} llsa_desc;

/* Opaque and host-side.  The level table and buffer layout never change after creation.  Unless
   desc.single_stream is set, the first llsa_backward call made outside stream capture creates the
   plan's auxiliary stream and events on the current device (calls made under capture before that,
   or on another device, simply stay on the caller's stream); llsa_backward serialises its enqueue
   sequence per plan, so a plan may be shared by host threads. */
typedef struct llsa_plan_s llsa_plan_t;

/* Validate a problem and precompute its level table and buffer layout (host only). */
llsa_status llsa_plan(const llsa_desc *desc, llsa_plan_t **out);
void llsa_plan_destroy(llsa_plan_t *plan);

/* Bytes of device workspace llsa_forward (for_backward = 0) / llsa_backward (1) need.
   The backward workspace starts with the forward one (same offsets). */
size_t llsa_plan_workspace_bytes(const llsa_plan_t *plan, int for_backward);

/* Total bytes of the int32 `indices` buffer: I^(0) | I^(1) | ... | I^(L-1), level l
   stored as [batch, heads, n_{l+1}, K_l]. */
size_t llsa_plan_indices_bytes(const llsa_plan_t *plan);

/* Level l (0..L-1) of `indices`: rows per head, K_l, byte offset.  Returns L, or -1 on bad input. */
int32_t llsa_plan_level_info(const llsa_plan_t *plan, int32_t l, int64_t *rows, int32_t *K_l,
                             size_t *byte_offset);

/* Where pooled level l (1..L) of tensor t (0 = Q, 1 = K, 2 = V) lives in the workspace:
   [batch, heads, n_l, d] of desc.dtype.  Returns 0, or -1 on bad input. */
int32_t llsa_plan_pyramid_info(const llsa_plan_t *plan, int32_t tensor, int32_t l, int64_t *tokens,
                               size_t *byte_offset);

/* Key-major lists of level l (0..L-1) inside the backward workspace (Alg. 2's outputs):
   C: [batch*heads, n_{l+1} + 1] int32 offsets; Iq: [batch*heads, n_{l+1} * K_l] int32 query-block
   rows, ascending within a key.  Returns 0, or -1 on bad input. */
int32_t llsa_plan_csc_info(const llsa_plan_t *plan, int32_t l, size_t *C_byte_offset, size_t *Iq_byte_offset);

/*
 * Forward pass (Alg. 1 in full).
 *   Q, K, V   in : [batch, heads, N, d]
 *   O        out : [batch, heads, N, d]
 *   LSE      out : [batch, heads, N] fp32, natural-log logsumexp of the logits
 *                  (sm_scale and the l ln B weights included)
 *   indices  out : see llsa_plan_indices_bytes
 *   workspace    : >= llsa_plan_workspace_bytes(plan, 0); holds the pooled levels afterwards
 */
llsa_status llsa_forward(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *O,
                         float *LSE, int32_t *indices, void *workspace, void *hip_stream);

/*
 * Backward pass with the selection held fixed (Sec. 4.3): recomputes P from LSE and the
 * lists, key/value gradients through the transposed lists (Alg. 2) and through the pooled
 * coarse tokens (adjoint of the compression loop of Alg. 1).
 *   Q, K, V, O, LSE, indices in : as given to / produced by llsa_forward
 *   dO                       in : [batch, heads, N, d]
 *   dQ, dK, dV              out : [batch, heads, N, d]
 *   workspace                   : >= llsa_plan_workspace_bytes(plan, 1); see desc.bwd_repool
 */
llsa_status llsa_backward(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, const void *O,
                          const float *LSE, const int32_t *indices, const void *dO, void *dQ, void *dK,
                          void *dV, void *workspace, void *hip_stream);

/*
 * llsa_forward for callers that cannot allocate device memory or have none to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as
 * llsa_forward, except that the workspace (the pooled levels of Q, K, V) is a static device array inside the
 * library, LLSA_STATIC_WORKSPACE_BYTES on every GPU the library is used on, held until the process ends.
 * The call allocates and frees nothing.
 *   - LLSA_ERR_WORKSPACE if llsa_plan_workspace_bytes(plan, 0) > llsa_static_workspace_bytes(): checked on
 *     the host first, nothing is enqueued (the headline shape, 16 heads of 65536 tokens at d = 64, needs 25.6 MiB).
 *   - The first call on a device looks the array's address up on that device (hipGetSymbolAddress); make
 *     that call outside stream capture.
 *   - Every call on one GPU uses the same array: calls that overlap on a GPU (two streams, two host threads)
 *     race.  The array keeps the last call's pooled levels; nothing in it needs clearing, since a call writes
 *     every byte it reads.  llsa_backward cannot use it: set desc.bwd_repool = 1 and pass backward a
 *     workspace of its own.
 */
#define LLSA_STATIC_WORKSPACE_BYTES (32u << 20)
size_t llsa_static_workspace_bytes(void);
llsa_status llsa_forward_static(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *O,
                                float *LSE, int32_t *indices, void *hip_stream);

/*
 * Layer glue fused with the first compression step (Sec. 5.2, "Training Settings": RoPE and QK-Norm sit in front
 * of the attention layer; Alg. 1, compression loop).  One pass over the pre-norm Q and K writes the level-0
 * tensors the layer consumes and their level-1 means, so they are not read back for pooling; V is pooled as usual;
 * then every remaining pooled level is filled, exactly as llsa_pool would on (Qout, Kout, V).
 *   per token t (position within its head) and tensor X in {Q, K}:
 *     y[c]        = Xpre[c] / sqrt(mean_c(Xpre[c]^2) + eps) * gamma_X[c]              (QK-Norm: RMS norm over d)
 *     Xout[2i]    = y[2i] * cos[t][i] - y[2i+1] * sin[t][i]
 *     Xout[2i+1]  = y[2i] * sin[t][i] + y[2i+1] * cos[t][i]                           (RoPE on adjacent channel pairs)
 *   Qpre, Kpre, V  in : [batch, heads, N, d] of desc.dtype
 *   gamma_q, gamma_k in : [d] fp32;   cos_table, sin_table in : [N, d / 2] fp32, shared by all heads (the caller
 *                    fills them for its token order: 1-D positions, or the two axes of a pixel grid)
 *   Qout, Kout    out : [batch, heads, N, d] of desc.dtype (fp32 arithmetic, one rounding); may not alias the inputs
 *   workspace         : >= llsa_plan_workspace_bytes(plan, 0); holds the pooled levels of (Qout, Kout, V) afterwards
 * Follow it with llsa_forward_pooled.  Errors: LLSA_ERR_NULL; LLSA_ERR_BAD_SHAPE for eps < 0 or misaligned pointers.
 */
llsa_status llsa_qknorm_rope_pool(const llsa_plan_t *plan, const void *Qpre, const void *Kpre, const void *V,
                                  const float *gamma_q, const float *gamma_k, const float *cos_table,
                                  const float *sin_table, float eps, void *Qout, void *Kout, void *workspace,
                                  void *hip_stream);

/* llsa_forward without its compression loop (Alg. 1, selection and enrichment loops only): `workspace` already
   holds the pooled levels of Q, K, V, from llsa_qknorm_rope_pool or llsa_pool.  Same outputs as llsa_forward. */
llsa_status llsa_forward_pooled(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *O,
                                float *LSE, int32_t *indices, void *workspace, void *hip_stream);

/* ---- the steps of the path one by one (same kernels; used for step-wise parity checks) ---- */

/* Hierarchical compression (Alg. 1, first loop): fills the pooled levels 1..L of Q, K, V in `workspace`. */
llsa_status llsa_pool(const llsa_plan_t *plan, const void *Q, const void *K, const void *V, void *workspace,
                      void *hip_stream);

/* One level of hierarchical Top-K selection (Alg. 1, second loop) at level l (1..L), reading the
   pooled Q^(l), K^(l) from `workspace`.  parent = I^(l) [batch, heads, n_{l+1}, K_l] (ignored, may be
   NULL, when l = L); out = I^(l-1) [batch, heads, n_l, K_{l-1}]. */
llsa_status llsa_select_level(const llsa_plan_t *plan, int32_t l, const void *workspace, const int32_t *parent,
                              int32_t *out, void *hip_stream);

/* Attention over the gathered lists only (Alg. 1, third loop; Eq. 1-5), given pooled levels in
   `workspace` and `indices`. */
llsa_status llsa_attention(const llsa_plan_t *plan, const void *Q, const void *K, const void *V,
                           const int32_t *indices, const void *workspace, void *O, float *LSE, void *hip_stream);

/* Alg. 2 for every level: builds the key-major lists inside the backward workspace. */
llsa_status llsa_index_transpose(const llsa_plan_t *plan, const int32_t *indices, void *workspace, void *hip_stream);

/*
 * Index reordering for 2-D token grids (Sec. 5.1, "Index Reordering"), applied once per model, outside
 * llsa_forward / llsa_backward: N = W * W tokens of a W x W pixel grid in raster order, W a power of two.
 * inverse = 0: out[bh][t] = in[bh][y * W + x], where x / y are the even / odd bits of t, so that for every i
 * each aligned run of 4^i tokens is one aligned 2^i x 2^i patch of pixels (nested patches; the four quarters
 * of a patch in row-major order).  inverse = 1 undoes it: out[bh][y * W + x] = in[bh][t].
 *   in, out : device, [batch_heads, N, d] of `dtype`, contiguous, caller-owned, not overlapping
 * Errors: LLSA_ERR_NULL; LLSA_ERR_UNSUPPORTED for an unknown dtype; LLSA_ERR_BAD_SHAPE if N is not a power
 * of four, a row is not a multiple of 16 bytes, or the buffers overlap.  Nothing is enqueued on error.
 */
llsa_status llsa_reorder(int64_t batch_heads, int64_t N, int32_t d, int32_t dtype, int32_t inverse, const void *in,
                         void *out, void *hip_stream);

/* ---- key/value backward of level 0 alone, with its key-major lists built two ways (benchmark comparator) ----
 * Sec. 5.4, "Efficient Backward Implementation" (Fig. 4) compares the key/value backward on the lists of Alg. 2 with
 * the mask-based baseline of earlier Top-K methods: the indices are turned into a dense binary T x T block mask
 * (T = N / B) and the backward scans it to skip the unmarked blocks.  Both are here, in front of the same dK / dV
 * kernel:  via_mask = 0: Alg. 2 (count, scan, fill; O(T K));  via_mask = 1: zero the mask, mark the listed
 * (key block, query block) pairs, scan every key block's T bytes and append the marked query blocks (O(T^2)).
 *   Q, K, V, dO, LSE, indices in : as for llsa_backward (bf16 plans that run the MFMA kernels only)
 *   workspace                    : a backward workspace on which llsa_backward has run for these tensors (the call
 *                                  reads D = rowsum(dO * O) from it and overwrites level 0's lists)
 *   mask                         : device, llsa_kv_backward_mask_bytes(plan) bytes (via_mask = 1; else may be NULL)
 *   dK0, dV0                 out : [batch, heads, N, d]: the gradient reaching K and V through level 0 alone
 *                                  (without the share of the pooled levels)
 * Errors: LLSA_ERR_NULL, LLSA_ERR_BAD_SHAPE (alignment), LLSA_ERR_UNSUPPORTED (a plan on the portable kernels). */
size_t llsa_kv_backward_mask_bytes(const llsa_plan_t *plan);
llsa_status llsa_kv_backward_level0(const llsa_plan_t *plan, int32_t via_mask, const void *Q, const void *K, const void *V,
                                    const void *dO, const float *LSE, const int32_t *indices, void *mask,
                                    void *workspace, void *dK0, void *dV0, void *hip_stream);

/* ---- per-stage timing for benchmarks (Sec. 5.4 reports kernel-level speed; this is how it is read here) ----
 * Stages: 0 pool, 1 select, 2 attention forward, 3 D = rowsum(dO*O), 4 index transpose, 5 dQ,
 * 6 dK/dV of the coarse levels, 7 un-pooling, 8 dK/dV of level 0.
 * llsa_stage_timing_begin creates HIP events (host objects, no device memory); until
 * llsa_stage_timing_end, every llsa_forward / llsa_backward call brackets stage `stage` (-1: every stage)
 * with two events on its stream, for at most `max_calls` calls of each.  llsa_stage_timing_end waits for
 * the recorded events, adds the elapsed milliseconds of stage i into ms_sum[i] and the number of
 * brackets into brackets[i] (HOST arrays of llsa_stage_count() entries, overwritten), and destroys the
 * events.  Process-global, not thread-safe: a benchmarking aid, not part of the compute path. */
int32_t llsa_stage_count(void);
const char *llsa_stage_name(int32_t stage);
llsa_status llsa_stage_timing_begin(int32_t stage, int32_t max_calls);
llsa_status llsa_stage_timing_end(double *ms_sum, int32_t *brackets);

/* ---- measured peaks of this GPU, for roofline fractions against what the chip delivers and not only the data sheet ----
 * llsa_calibrate_mfma: `workgroups` workgroups of 4 waves, each wave 8 * iters bf16 MFMAs of 16 x 16 x 32 (16384 FLOP
 * each) on registers only; the caller times the launch: FLOP = workgroups * 4 * 8 * iters * 16384.  `out`: device,
 * at least 4 bytes, never written.  llsa_calibrate_copy: a plain copy of `bytes` (a multiple of 16) device bytes,
 * 16 per thread; traffic = 2 * bytes. */
llsa_status llsa_calibrate_mfma(float *out, int32_t iters, int32_t workgroups, void *hip_stream);
llsa_status llsa_calibrate_copy(const void *src, void *dst, int64_t bytes, void *hip_stream);

const char *llsa_status_string(llsa_status s);

#ifdef __cplusplus
}
#endif
#endif /* LLSA_H */
