// Attention forward over the gathered lists on bf16 MFMA (B = 16, 32 or 64, d = 64 or 128): Alg. 1's attention loop
// with Eq. 1-5 evaluated tile by tile with an online softmax.
//
// One wave owns one tile of 16 queries.  Per tile of two 16-token key blocks it computes
//   S^T = K Q^T   (A = key rows straight from global memory, B = the query block held in registers),
// so every lane ends up with 4 keys x 1 query of S^T; the softmax statistics of a query are then a
// reduction inside the lane plus two cross-row steps, and the probabilities already sit in the register
// layout the second product wants as its B operand:
//   O^T += V^T P^T (A = V^T read from LDS with the transposing 64-bit read, B = P^T).
// V tiles are staged per wave in LDS (row-major, padded rows) because the second product contracts over
// keys while V is stored with d contiguous.  The running row sum is kept per lane and combined across
// the four row groups once at the end; accumulators are rescaled only in tiles that raise a row maximum.
#include "mfma_common.h"

namespace llsa {

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 4 : 2))) attn_fwd_mfma_kernel(LevelTable t, const uint16_t *__restrict__ Q,
                                                             uint16_t *__restrict__ O, float *__restrict__ LSE,
                                                             int64_t N, int64_t total_wgs) {
    constexpr int KS = D / 32;            // MFMA steps over d for S^T
    constexpr int NT = D / 16;            // 16-wide d tiles of O^T
    constexpr int STRIDE = D * 2 + 32;    // bytes per key row in LDS (padding spreads the rows over the banks)
    constexpr int VCH = D / 16;           // 16-byte chunks of a 32-key V tile per lane
    constexpr int PARTS = D / 8;          // 16-byte chunks per key row
    constexpr int KPU = 64 / PARTS;       // key rows covered by one chunk round of the wave
    __shared__ __attribute__((aligned(16))) char vlds[4][32 * STRIDE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t nblk = N >> 4;                                     // fine query blocks per head
    const int64_t fb = xcd_contiguous(blockIdx.x, total_wgs) * 4 + wave;
    const int64_t bh = fb / nblk, blk = fb % nblk;                  // nblk % 4 == 0: a workgroup stays in one head
    const int i16 = lane & 15, g = lane >> 4;
    char *my = vlds[wave];

    bf16x8 qop[KS];
    {
        const uint16_t *qrow = Q + (bh * N + blk * 16 + i16) * D + g * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) qop[s] = ld_bf16x8(qrow + 32 * s);
    }
    f32x4 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, lsum = 0.f;                                 // lsum: this lane's share of the row sum
    const float sc2 = t.scale * kLog2e;
    const int nb = t.bseg[t.nlev];                                   // key blocks in the list

    BlockTable tab;
    tab.fill(t, bh, blk, 0, 0, lane, D);

    // per-lane byte offsets inside a block (row-wise operand load / 16-byte staging chunks)
    const int koff = (i16 * D + g * 8) * 2;
    int voff[VCH];
#pragma unroll
    for (int u = 0; u < VCH; ++u) voff[u] = (((lane / PARTS + KPU * u) & 15) * D + (lane % PARTS) * 8) * 2;

    bf16x8 kop[2][KS];
    u32x4 vreg[VCH];
    float bias2[2];
    int cnt[2];

    auto load_tile = [&](int j0) {                                   // blocks j0 and j0 + 1 (j0 even)
        if (j0 > 0 && (j0 & 63) == 0) tab.fill(t, bh, blk, 0, j0 >> 6, lane, D);
        const char *kp[2], *vp[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int j = (j0 + h < nb) ? j0 + h : j0;              // an absent second half re-reads the first
            kp[h] = tab.K(j & 63);
            vp[h] = tab.V(j & 63);
            cnt[h] = (j0 + h < nb) ? tab.count(j & 63) : 0;
            bias2[h] = tab.bias(j & 63);
            const int last = max(cnt[h], 1) - 1;                     // rows past a ragged end re-read the last row
            const int ko = cnt[h] < 16 ? (min(i16, last) * D + g * 8) * 2 : koff;
#pragma unroll
            for (int s = 0; s < KS; ++s) kop[h][s] = ld_bf16x8(kp[h] + ko + 64 * s);
        }
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            const int h = (KPU * u) >> 4;                            // which half this chunk round belongs to
            const int last = max(cnt[h], 1) - 1;
            const int vo = cnt[h] < 16 ? (min((lane / PARTS + KPU * u) & 15, last) * D + (lane % PARTS) * 8) * 2 : voff[u];
            vreg[u] = *reinterpret_cast<const u32x4 *>(vp[h] + vo);
        }
    };

    load_tile(0);
    for (int j0 = 0; j0 < nb; j0 += 2) {
        // stage this tile's V rows; LDS operations of one wave complete in order, the barriers only pin
        // the compiler's schedule
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            const int key = lane / PARTS + KPU * u, part = lane % PARTS;
            *reinterpret_cast<u32x4 *>(my + key * STRIDE + part * 16) = vreg[u];
        }
        __builtin_amdgcn_wave_barrier();

        f32x4 s[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) s[h] = mfma16(kop[h][ks], qop[ks], s[h]);
        }
        const float b2[2] = {bias2[0], bias2[1]};
        const int c[2] = {cnt[0], cnt[1]};
        if (j0 + 2 < nb) load_tile(j0 + 2);                          // next tile's loads fly during the math

        float mx = -INFINITY;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s[h][r] = fmaf(s[h][r], sc2, b2[h]);
                mx = fmaxf(mx, s[h][r]);
            }
        if (c[0] < 16 || c[1] < 16) {                                // ragged or absent block: mask and redo the max
            mx = -INFINITY;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (4 * g + r >= c[h]) s[h][r] = -INFINITY;
                    mx = fmaxf(mx, s[h][r]);
                }
        }
        mx = rows_max(mx);
        if (__builtin_amdgcn_ballot_w64(mx > m) != 0) {              // some row's maximum rose: rescale
            const float m_new = fmaxf(m, mx);
            const float alpha = __builtin_amdgcn_exp2f(m - m_new);
            lsum *= alpha;
#pragma unroll
            for (int n = 0; n < NT; ++n)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[n][r] *= alpha;
            m = m_new;
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                s[h][r] = __builtin_amdgcn_exp2f(s[h][r] - m);
                lsum += s[h][r];
            }
        const bf16x8 pop = pack8(s[0], s[1]);

        const char *base = my + (4 * g + (i16 >> 2)) * STRIDE + (i16 & 3) * 8;
#pragma unroll
        for (int n = 0; n < NT; ++n)
            acc[n] = mfma16(lds_tr_pair(base + n * 32, base + 16 * STRIDE + n * 32), pop, acc[n]);
    }

    lsum = rows_sum(lsum);
    const float inv = 1.f / lsum;
    uint16_t *orow = O + (bh * N + blk * 16 + i16) * D + 4 * g;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        u32x2 w;
        w[0] = pack_bf16(acc[n][0] * inv, acc[n][1] * inv);
        w[1] = pack_bf16(acc[n][2] * inv, acc[n][3] * inv);
        *reinterpret_cast<u32x2 *>(orow + n * 16) = w;
    }
    if (g == 0) LSE[bh * N + blk * 16 + i16] = (m + __builtin_amdgcn_logf(lsum)) * kLn2;
}

hipError_t launch_attn_fwd_mfma(const Plan &p, const LevelTable &t, const void *Q, void *O, float *LSE,
                                hipStream_t s) {
    if (p.N % 256 == 0 && (p.Kl[0] << (p.lb - 4)) <= 64) return launch_attn_fwd_shared(p, t, Q, O, LSE, s);
    const int64_t wgs = (int64_t)p.bh * (p.N / 64);                  // 4 query blocks per workgroup
    dim3 grid((unsigned)wgs);
    if (p.d == 64)
        attn_fwd_mfma_kernel<64><<<grid, 256, 0, s>>>(t, (const uint16_t *)Q, (uint16_t *)O, LSE, p.N, wgs);
    else
        attn_fwd_mfma_kernel<128><<<grid, 256, 0, s>>>(t, (const uint16_t *)Q, (uint16_t *)O, LSE, p.N, wgs);
    return hipGetLastError();
}

}  // namespace llsa
