/* Calls every function of the CPU oracle once on small shapes with exactly sized buffers, for a build with
 * -fsanitize=address,undefined (tests/test_oracle_sanitize.py): an out-of-bounds index or an overflow anywhere in
 * the oracle shows up as a sanitizer report.  Shapes: N = 144, B = 4 and 6 (a ragged top level), K larger than the
 * rows of the top level, every enrichment depth, a row sub-range. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void llsa_oracle_pool(const float *x, int64_t n_out, int d, int B, int round_bf16, float *y);
int llsa_oracle_select(const float *Ql, const float *Kl, int64_t n_l, int d, int B, const int32_t *parent, int Kp,
                       int Kout, int32_t *out, double *margin);
int64_t llsa_oracle_list_len(int64_t N, int B, int K, int L, int Le);
int64_t llsa_oracle_kv_list(const int32_t *idx, int64_t N, int B, int K, int L, int Le, int64_t i, int32_t *lev,
                            int64_t *tok);
int llsa_oracle_attn_fwd(const double *Q, const double *Kpyr, const double *Vpyr, const int32_t *idx, int64_t N, int d,
                         int B, int K, int L, int Le, int reweight, double scale, int64_t q_begin, int64_t q_end,
                         double *O, double *LSE);
int llsa_oracle_attn_bwd(const double *Q, const double *Kpyr, const double *Vpyr, const int32_t *idx, const double *dO,
                         int64_t N, int d, int B, int K, int L, int Le, int reweight, double scale, int64_t q_begin,
                         int64_t q_end, double *dQ, double *dKpyr, double *dVpyr);
void llsa_oracle_unpool(double *gpyr, int64_t N, int d, int B, int L, double *gx);
void llsa_oracle_transpose(const int32_t *I, int64_t T_rows, int K, int64_t T_keys, int32_t *Iq, int32_t *C);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static float rnd(void) { state = state * 6364136223846793005ull + 1442695040888963407ull; return (float)((state >> 40) / 16777216.0 - 0.5); }

static int walk(int64_t N, int d, int B, int K, int L)
{
    int64_t n[8], tot = 0, ntok = N;
    int Kl[8];
    for (int l = 0; l <= L; ++l) { n[l] = ntok; tot += ntok; ntok /= B; }
    for (int l = 0; l < L; ++l) Kl[l] = (int)(n[l + 1] < K ? n[l + 1] : K);
    float *lev[3][8];
    for (int x = 0; x < 3; ++x) {
        lev[x][0] = (float *)malloc(sizeof(float) * (size_t)(N * d));
        for (int64_t i = 0; i < N * d; ++i) lev[x][0][i] = rnd();
        for (int l = 1; l <= L; ++l) {
            lev[x][l] = (float *)malloc(sizeof(float) * (size_t)(n[l] * d));
            llsa_oracle_pool(lev[x][l - 1], n[l], d, B, x != 2, lev[x][l]);
        }
    }
    int64_t ient = 0, ioff[8];
    for (int l = 0; l < L; ++l) { ioff[l] = ient; ient += n[l + 1] * Kl[l]; }
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)ient);
    for (int l = L; l >= 1; --l) {
        double *margin = (double *)malloc(sizeof(double) * (size_t)n[l]);
        const int32_t *parent = (l == L) ? NULL : idx + ioff[l];
        if (llsa_oracle_select(lev[0][l], lev[1][l], n[l], d, B, parent, l == L ? 0 : Kl[l], Kl[l - 1], idx + ioff[l - 1], margin))
            return 1;
        free(margin);
    }
    double *Q = (double *)malloc(sizeof(double) * (size_t)(N * d)), *dO = (double *)malloc(sizeof(double) * (size_t)(N * d));
    double *Kp = (double *)malloc(sizeof(double) * (size_t)(tot * d)), *Vp = (double *)malloc(sizeof(double) * (size_t)(tot * d));
    for (int64_t i = 0; i < N * d; ++i) { Q[i] = lev[0][0][i]; dO[i] = rnd(); }
    int64_t off = 0;
    for (int l = 0; l <= L; ++l) {
        for (int64_t i = 0; i < n[l] * d; ++i) { Kp[off * d + i] = lev[1][l][i]; Vp[off * d + i] = lev[2][l][i]; }
        off += n[l];
    }
    double *O = (double *)malloc(sizeof(double) * (size_t)(N * d)), *LSE = (double *)malloc(sizeof(double) * (size_t)N);
    double *dQ = (double *)malloc(sizeof(double) * (size_t)(N * d));
    double *dKp = (double *)malloc(sizeof(double) * (size_t)(tot * d)), *dVp = (double *)malloc(sizeof(double) * (size_t)(tot * d));
    double *gx = (double *)malloc(sizeof(double) * (size_t)(N * d));
    for (int Le = 0; Le <= L; ++Le) {
        int64_t cap = llsa_oracle_list_len(N, B, K, L, Le);
        int32_t *lv = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap);
        int64_t *tk = (int64_t *)malloc(sizeof(int64_t) * (size_t)cap);
        if (llsa_oracle_kv_list(idx, N, B, K, L, Le, N / B - 1, lv, tk) != cap) return 2;
        free(lv); free(tk);
        for (int rw = 0; rw <= 2; ++rw)
            if (llsa_oracle_attn_fwd(Q, Kp, Vp, idx, N, d, B, K, L, Le, rw, 0.25, 0, N, O, LSE)) return 3;
        if (llsa_oracle_attn_fwd(Q, Kp, Vp, idx, N, d, B, K, L, Le, 1, 0.25, N - 3, N, O, LSE)) return 4;
        if (llsa_oracle_attn_bwd(Q, Kp, Vp, idx, dO, N, d, B, K, L, Le, 1, 0.25, 0, N, dQ, dKp, dVp)) return 5;
        if (llsa_oracle_attn_bwd(Q, Kp, Vp, idx, dO, N, d, B, K, L, Le, 0, 0.25, 5, 9, dQ, dKp, dVp)) return 6;
        llsa_oracle_unpool(dKp, N, d, B, L, gx);
        for (int64_t i = 0; i < N * d; ++i) if (!isfinite(gx[i]) || !isfinite(O[i])) return 7;
    }
    for (int l = 0; l < L; ++l) {
        int32_t *Iq = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n[l + 1] * Kl[l]));
        int32_t *C = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n[l + 1] + 1));
        llsa_oracle_transpose(idx + ioff[l], n[l + 1], Kl[l], n[l + 1], Iq, C);
        if (C[n[l + 1]] != n[l + 1] * Kl[l]) return 8;
        free(Iq); free(C);
    }
    for (int x = 0; x < 3; ++x) for (int l = 0; l <= L; ++l) free(lev[x][l]);
    free(idx); free(Q); free(dO); free(Kp); free(Vp); free(O); free(LSE); free(dQ); free(dKp); free(dVp); free(gx);
    return 0;
}

int main(void)
{
    int rc;
    if ((rc = walk(144, 8, 4, 2, 2))) { printf("walk 1 failed: %d\n", rc); return 1; }      /* 144 / 36 / 9 */
    if ((rc = walk(144, 8, 6, 8, 2))) { printf("walk 2 failed: %d\n", rc); return 1; }      /* 144 / 24 / 4: K above the top rows */
    if ((rc = walk(256, 16, 4, 3, 3))) { printf("walk 3 failed: %d\n", rc); return 1; }     /* 256 / 64 / 16 / 4 */
    printf("oracle walk ok\n");
    return 0;
}
