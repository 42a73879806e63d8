/*
 * CPU oracle for Log-linear Sparse Attention (LLSA).
 *
 * TEST INFRASTRUCTURE ONLY.  A plain, slow, single-threaded-per-head
 * implementation of the method as the paper defines it, used to check the
 * GPU library.  It shares no code with the GPU path and must never be called
 * from it.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may load this file.
 *
 * What follows the paper, passage by passage:
 *   - pyramid         : Alg. 1 "Hierarchical Compression" loop; Sec. 4.1
 *                       "Hierarchical Compression" (mean over B consecutive
 *                       tokens, each level pooled from the previous one).
 *   - selection       : Alg. 1 "Hierarchical Top-K Selection" loop; Sec. 4.1
 *                       "Hierarchical Top-K Selection" (dense scores at the
 *                       coarsest level, K*B gathered candidates below it).
 *   - kv list         : Alg. 1 "Hierarchical KV Enrichment" loop; Sec. 4.1
 *                       "Hierarchical KV Enrichment" and "KV Reweighting".
 *   - attention       : Eq. 1-5 (softmax attention restricted to the list).
 *   - backward        : standard softmax-attention gradients over the list
 *                       (Sec. 4.3, key-major accumulation is an
 *                       implementation matter; here the sums are written
 *                       query by query), then the adjoint of mean pooling.
 *   - index transpose : Alg. 2 (count, cumulative sum, fill).
 *
 * Readings taken where the paper is silent (all 0-based):
 *   - K_l = min(K, n_{l+1}) entries per row of I^(l); rows sorted ascending.
 *   - Top-K order: larger score first, equal scores -> lower key id first.
 *   - scores: unscaled fp32 dot product accumulated with fused multiply-add
 *     over channels 0..d-1 in order (the selection decides an integer, so the
 *     precision is fixed: fp32); an fp64 shadow reports the K-th/(K+1)-th gap.
 *   - pooling: fp32 sum of the B children in ascending order, divided by B,
 *     rounded (nearest-even) to the I/O type when that type is bf16.
 *   - reweighting: a level-l token counts as B^l copies, i.e. its logit gets
 *     + l*ln(B).  mode 0 = no weight, mode 1 = this reading (default),
 *     mode 2 = the literal reading of Alg. 1 (K and V multiplied by B^l;
 *     forward only, kept to show the difference).
 *   - fine query block i uses row i / B^l of I^(l); no de-duplication across
 *     levels; level L (if enriched) contributes all n_L tokens.
 *   - attention and gradients are evaluated in fp64.
 *
 * parity unpinned: the near-tie margin rule (a convention of this build).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ utils */

static float round_to_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return x; /* inf / nan untouched */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&x, &u, 4);
    return x;
}

static int64_t ipow(int64_t b, int e)
{
    int64_t r = 1;
    while (e-- > 0) r *= b;
    return r;
}

/* tokens at level l */
static int64_t level_tokens(int64_t N, int B, int l) { return N / ipow(B, l); }

/* offset (in tokens) of level l inside a concatenated pyramid [n_0 | n_1 | ... | n_L] */
static int64_t pyr_offset(int64_t N, int B, int l)
{
    int64_t off = 0;
    for (int j = 0; j < l; ++j) off += level_tokens(N, B, j);
    return off;
}

static int k_of_level(int64_t N, int B, int K, int l)
{
    int64_t blocks = level_tokens(N, B, l + 1); /* key blocks at level l */
    return (int)(blocks < K ? blocks : K);
}

/* offset (in int32 entries) of I^(l) inside the concatenation I^(0) | I^(1) | ... | I^(L-1) */
static int64_t idx_offset(int64_t N, int B, int K, int l)
{
    int64_t off = 0;
    for (int j = 0; j < l; ++j) off += level_tokens(N, B, j + 1) * k_of_level(N, B, K, j);
    return off;
}

/* ---------------------------------------------------------------- pyramid */

/* One pooling step: y[t] = mean_{r<B} x[t*B + r], t < n_out.  x: [n_out*B, d]. */
void llsa_oracle_pool(const float *x, int64_t n_out, int d, int B, int round_bf16, float *y)
{
    for (int64_t t = 0; t < n_out; ++t)
        for (int c = 0; c < d; ++c) {
            float s = 0.0f;
            for (int r = 0; r < B; ++r) s = s + x[(t * B + r) * d + c];
            s = s / (float)B;
            y[t * d + c] = round_bf16 ? round_to_bf16(s) : s;
        }
}

/* ---------------------------------------------------------------- select  */

typedef struct {
    float s;
    double s64;
    int32_t id;
} cand_t;

static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

static int id_cmp(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Selection at one level l (1 <= l <= L).
 *   Ql, Kl   : level-l queries / keys, [n_l, d]
 *   parent   : NULL at the coarsest level (candidates = all n_l tokens);
 *              else I^(l), [n_l / B, Kp]: key-block ids at level l
 *   out      : I^(l-1), [n_l, Kout], each row sorted ascending
 *   margin   : optional [n_l]; relative gap between the Kout-th and the
 *              (Kout+1)-th candidate measured on the fp64 scores
 *              (+inf when every candidate is taken)
 */
int llsa_oracle_select(const float *Ql, const float *Kl, int64_t n_l, int d, int B,
                       const int32_t *parent, int Kp, int Kout, int32_t *out, double *margin)
{
    int64_t ncand = parent ? (int64_t)Kp * B : n_l;
    if (Kout > ncand) return 1;
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)ncand);
    if (!cand) return 2;
    for (int64_t i = 0; i < n_l; ++i) {
        const float *q = Ql + i * d;
        for (int64_t p = 0; p < ncand; ++p) {
            int64_t id = parent ? (int64_t)parent[(i / B) * Kp + p / B] * B + p % B : p;
            const float *k = Kl + id * d;
            float s = 0.0f;
            double s64 = 0.0;
            for (int c = 0; c < d; ++c) {
                s = fmaf(q[c], k[c], s);
                s64 += (double)q[c] * (double)k[c];
            }
            cand[p].s = s;
            cand[p].s64 = s64;
            cand[p].id = (int32_t)id;
        }
        qsort(cand, (size_t)ncand, sizeof(cand_t), cand_cmp);
        for (int k = 0; k < Kout; ++k) out[i * Kout + k] = cand[k].id;
        qsort(out + i * Kout, (size_t)Kout, sizeof(int32_t), id_cmp);
        if (margin) {
            if (Kout == ncand) {
                margin[i] = INFINITY;
            } else {
                /* gap on the fp64 scores between the weakest taken and the strongest left out */
                double lo = INFINITY, hi = -INFINITY;
                for (int64_t p = 0; p < ncand; ++p) {
                    if (p < Kout) { if (cand[p].s64 < lo) lo = cand[p].s64; }
                    else          { if (cand[p].s64 > hi) hi = cand[p].s64; }
                }
                double den = fmax(fabs(lo), fabs(hi));
                margin[i] = den > 0.0 ? (lo - hi) / den : 0.0;
            }
        }
    }
    free(cand);
    return 0;
}

/* ----------------------------------------------------------------- kv list */

/*
 * The (level, token) list fine query block i attends to.
 *   idx   : I^(0) | ... | I^(L-1) concatenated, I^(l): [n_{l+1}, K_l]
 *   lev, tok : outputs, capacity >= llsa_oracle_list_len()
 * returns the number of entries.
 */
int64_t llsa_oracle_list_len(int64_t N, int B, int K, int L, int Le)
{
    int64_t m = 0;
    for (int l = 0; l <= Le; ++l)
        m += (l < L) ? (int64_t)k_of_level(N, B, K, l) * B : level_tokens(N, B, L);
    return m;
}

int64_t llsa_oracle_kv_list(const int32_t *idx, int64_t N, int B, int K, int L, int Le,
                            int64_t i, int32_t *lev, int64_t *tok)
{
    int64_t m = 0;
    for (int l = 0; l <= Le; ++l) {
        if (l < L) {
            int Kl = k_of_level(N, B, K, l);
            int64_t row = i / ipow(B, l);
            const int32_t *I = idx + idx_offset(N, B, K, l) + row * Kl;
            for (int k = 0; k < Kl; ++k)
                for (int u = 0; u < B; ++u) {
                    lev[m] = l;
                    tok[m] = (int64_t)I[k] * B + u;
                    ++m;
                }
        } else {
            int64_t nL = level_tokens(N, B, L);
            for (int64_t c = 0; c < nL; ++c) {
                lev[m] = l;
                tok[m] = c;
                ++m;
            }
        }
    }
    return m;
}

/* --------------------------------------------------------------- attention */

static double dot64(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += a[c] * b[c];
    return s;
}

/* logits of one query over its list; returns logsumexp */
static double row_logits(const double *q, const double *Kpyr, int64_t N, int d, int B, int reweight,
                         double scale, int64_t m, const int32_t *lev, const int64_t *tok, double *z)
{
    double lnB = log((double)B), zmax = -INFINITY;
    for (int64_t j = 0; j < m; ++j) {
        const double *k = Kpyr + (pyr_offset(N, B, lev[j]) + tok[j]) * d;
        double s = scale * dot64(q, k, d);
        if (reweight == 1) s += lev[j] * lnB;
        else if (reweight == 2) s *= (double)ipow(B, lev[j]);
        z[j] = s;
        if (s > zmax) zmax = s;
    }
    double sum = 0.0;
    for (int64_t j = 0; j < m; ++j) sum += exp(z[j] - zmax);
    return zmax + log(sum);
}

/*
 * Forward over query rows [q_begin, q_end).
 *   Q     : [N, d] fp64;  Kpyr, Vpyr : concatenated pyramids [sum_l n_l, d] fp64
 *   O     : [N, d] fp64 (only the requested rows are written); LSE : [N]
 */
int llsa_oracle_attn_fwd(const double *Q, const double *Kpyr, const double *Vpyr, const int32_t *idx,
                         int64_t N, int d, int B, int K, int L, int Le, int reweight, double scale,
                         int64_t q_begin, int64_t q_end, double *O, double *LSE)
{
    int64_t cap = llsa_oracle_list_len(N, B, K, L, Le);
    int32_t *lev = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
    int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)cap);
    double *z = (double *)malloc(sizeof(double) * (size_t)cap);
    if (!lev || !tok || !z) return 2;
    for (int64_t q = q_begin; q < q_end; ++q) {
        int64_t m = llsa_oracle_kv_list(idx, N, B, K, L, Le, q / B, lev, tok);
        double lse = row_logits(Q + q * d, Kpyr, N, d, B, reweight, scale, m, lev, tok, z);
        double *o = O + q * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int64_t j = 0; j < m; ++j) {
            double p = exp(z[j] - lse);
            const double *v = Vpyr + (pyr_offset(N, B, lev[j]) + tok[j]) * d;
            double w = (reweight == 2) ? (double)ipow(B, lev[j]) : 1.0;
            for (int c = 0; c < d; ++c) o[c] += p * w * v[c];
        }
        LSE[q] = lse;
    }
    free(lev); free(tok); free(z);
    return 0;
}

/*
 * Backward with the indices held fixed (reweight modes 0 and 1).
 *   dO            : [N, d]
 *   dQ            : [N, d]            (overwritten)
 *   dKpyr, dVpyr  : [sum_l n_l, d]    (overwritten) gradients w.r.t. every
 *                   pyramid level taken as an independent variable
 *   q_begin,q_end : only these query rows contribute (the whole sum is
 *                   0..N; a sub-range gives that range's share of dK, dV
 *                   and its rows of dQ, the other rows of dQ stay zero)
 */
int llsa_oracle_attn_bwd(const double *Q, const double *Kpyr, const double *Vpyr, const int32_t *idx,
                         const double *dO, int64_t N, int d, int B, int K, int L, int Le, int reweight,
                         double scale, int64_t q_begin, int64_t q_end, double *dQ, double *dKpyr, double *dVpyr)
{
    if (reweight != 0 && reweight != 1) return 1;
    int64_t cap = llsa_oracle_list_len(N, B, K, L, Le);
    int64_t tot = pyr_offset(N, B, L + 1);
    int32_t *lev = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
    int64_t *tok = (int64_t *)malloc(sizeof(int64_t) * (size_t)cap);
    double *z = (double *)malloc(sizeof(double) * (size_t)cap);
    double *dp = (double *)malloc(sizeof(double) * (size_t)cap);
    if (!lev || !tok || !z || !dp) return 2;
    memset(dQ, 0, sizeof(double) * (size_t)(N * d));
    memset(dKpyr, 0, sizeof(double) * (size_t)(tot * d));
    memset(dVpyr, 0, sizeof(double) * (size_t)(tot * d));
    for (int64_t q = q_begin; q < q_end; ++q) {
        int64_t m = llsa_oracle_kv_list(idx, N, B, K, L, Le, q / B, lev, tok);
        const double *qv = Q + q * d, *go = dO + q * d;
        double lse = row_logits(qv, Kpyr, N, d, B, reweight, scale, m, lev, tok, z);
        double delta = 0.0; /* sum_j p_j dp_j  (= dO . O) */
        for (int64_t j = 0; j < m; ++j) {
            z[j] = exp(z[j] - lse); /* z now holds p */
            dp[j] = dot64(go, Vpyr + (pyr_offset(N, B, lev[j]) + tok[j]) * d, d);
            delta += z[j] * dp[j];
        }
        for (int64_t j = 0; j < m; ++j) {
            int64_t row = pyr_offset(N, B, lev[j]) + tok[j];
            double p = z[j], ds = p * (dp[j] - delta);
            const double *k = Kpyr + row * d;
            double *gk = dKpyr + row * d, *gv = dVpyr + row * d, *gq = dQ + q * d;
            for (int c = 0; c < d; ++c) {
                gq[c] += scale * ds * k[c];
                gk[c] += scale * ds * qv[c];
                gv[c] += p * go[c];
            }
        }
    }
    free(lev); free(tok); free(z); free(dp);
    return 0;
}

/*
 * Adjoint of the pyramid: fold the gradients of the pooled levels back into
 * level 0.  gpyr: [sum_l n_l, d] (modified in place); gx: [N, d] result.
 * level l-1 token t*B + r receives (1/B) of level-l token t.
 */
void llsa_oracle_unpool(double *gpyr, int64_t N, int d, int B, int L, double *gx)
{
    for (int l = L; l >= 1; --l) {
        int64_t n = level_tokens(N, B, l);
        double *src = gpyr + pyr_offset(N, B, l) * d, *dst = gpyr + pyr_offset(N, B, l - 1) * d;
        for (int64_t t = 0; t < n; ++t)
            for (int r = 0; r < B; ++r)
                for (int c = 0; c < d; ++c) dst[(t * B + r) * d + c] += src[t * d + c] / (double)B;
    }
    memcpy(gx, gpyr, sizeof(double) * (size_t)(N * d));
}

/* --------------------------------------------------------- index transpose */

/*
 * Alg. 2: row-major lists I [T_rows, K] over T_keys key blocks -> key-major
 * (Iq [T_rows*K], C [T_keys+1]).  Within a key the query rows come out in
 * ascending order because the fill loop visits rows in ascending order.
 */
void llsa_oracle_transpose(const int32_t *I, int64_t T_rows, int K, int64_t T_keys, int32_t *Iq, int32_t *C)
{
    int32_t *fill = (int32_t *)calloc((size_t)T_keys, sizeof(int32_t));
    for (int64_t j = 0; j <= T_keys; ++j) C[j] = 0;
    for (int64_t i = 0; i < T_rows; ++i)           /* count */
        for (int k = 0; k < K; ++k) C[I[i * K + k] + 1] += 1;
    for (int64_t j = 0; j < T_keys; ++j) C[j + 1] += C[j]; /* cumulative sum */
    for (int64_t i = 0; i < T_rows; ++i)           /* fill */
        for (int k = 0; k < K; ++k) {
            int32_t key = I[i * K + k];
            Iq[C[key] + fill[key]] = (int32_t)i;
            fill[key] += 1;
        }
    free(fill);
}
