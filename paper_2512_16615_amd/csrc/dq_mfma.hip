// dQ of the gathered-list attention on bf16 MFMA (B = 16, 32 or 64, d = 64 or 128), Sec. 4.3: query-major, the
// same list walk as the forward, P recomputed from the saved logsumexp.
// With P = exp(z - LSE), dP = dO V^T, dS = P o (dP - D), D = rowsum(dO o O):  dQ = scale dS K.
//
// One wave per tile of 16 queries.  Per tile of two 16-token key tiles:
//   S^T = K Q^T, dP^T = V dO^T  (lane: 4 keys x 1 query)  ->  dS^T  ->  dQ^T += K^T dS^T.
// K tiles are staged in the wave's LDS region and read twice (row-wise for S^T, transposed for dQ^T);
// V rows go straight from global memory into the A operand.  The kernel also produces D for its 16
// queries (one pass over O and dO, which it holds anyway) and stores it for the key-major kernels.
#include "mfma_common.h"

namespace llsa {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

template <int D>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(D == 64 ? 4 : 2))) dq_mfma_kernel(LevelTable t, const uint16_t *__restrict__ Q,
                                                       const uint16_t *__restrict__ O, const uint16_t *__restrict__ dO,
                                                       const float *__restrict__ LSE, float *__restrict__ Dsum,
                                                       uint16_t *__restrict__ dQ, int64_t N, int64_t total_wgs) {
    constexpr int KS = D / 32, NT = D / 16, STRIDE = D * 2 + 32, VCH = D / 16, PARTS = D / 8, KPU = 64 / PARTS;
    __shared__ __attribute__((aligned(16))) char klds[4][32 * STRIDE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t nblk = N >> 4;
    const int64_t fb = xcd_contiguous(blockIdx.x, total_wgs) * 4 + wave;
    const int64_t bh = fb / nblk, blk = fb % nblk;
    const int i16 = lane & 15, g = lane >> 4;
    char *my = klds[wave];

    const int64_t qrow = bh * N + blk * 16 + i16;
    bf16x8 qop[KS], gop[KS];
    float delta = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        qop[s] = ld_bf16x8(Q + qrow * D + g * 8 + 32 * s);
        const u32x4 gw = *reinterpret_cast<const u32x4 *>(dO + qrow * D + g * 8 + 32 * s);
        const u32x4 ow = *reinterpret_cast<const u32x4 *>(O + qrow * D + g * 8 + 32 * s);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            delta = fmaf(bf16_lo(gw[e]), bf16_lo(ow[e]), delta);
            delta = fmaf(bf16_hi(gw[e]), bf16_hi(ow[e]), delta);
        }
        union { u32x4 u; bf16x8 v; } cv;
        cv.u = gw;
        gop[s] = cv.v;
    }
    delta = rows_sum(delta);
    if (g == 0) Dsum[qrow] = delta;
    const float lse2 = LSE[qrow] * kLog2e;
    const float sc2 = t.scale * kLog2e;
    f32x4 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nb = t.bseg[t.nlev];

    BlockTable tab;
    tab.fill(t, bh, blk, 0, 0, lane, D);
    const int koff = (i16 * D + g * 8) * 2;
    int voff[VCH];
#pragma unroll
    for (int u = 0; u < VCH; ++u) voff[u] = (((lane / PARTS + KPU * u) & 15) * D + (lane % PARTS) * 8) * 2;

    bf16x8 vop[2][KS];
    u32x4 kreg[VCH];
    float bias2[2];
    int cnt[2];

    auto load_tile = [&](int j0) {
        if (j0 > 0 && (j0 & 63) == 0) tab.fill(t, bh, blk, 0, j0 >> 6, lane, D);
        const char *kp[2], *vp[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int j = (j0 + h < nb) ? j0 + h : j0;
            kp[h] = tab.K(j & 63);
            vp[h] = tab.V(j & 63);
            cnt[h] = (j0 + h < nb) ? tab.count(j & 63) : 0;
            bias2[h] = tab.bias(j & 63);
            const int last = max(cnt[h], 1) - 1;
            const int vo = cnt[h] < 16 ? (min(i16, last) * D + g * 8) * 2 : koff;
#pragma unroll
            for (int s = 0; s < KS; ++s) vop[h][s] = ld_bf16x8(vp[h] + vo + 64 * s);
        }
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            const int h = (KPU * u) >> 4;
            const int last = max(cnt[h], 1) - 1;
            const int ko = cnt[h] < 16 ? (min((lane / PARTS + KPU * u) & 15, last) * D + (lane % PARTS) * 8) * 2 : voff[u];
            kreg[u] = *reinterpret_cast<const u32x4 *>(kp[h] + ko);
        }
    };

    load_tile(0);
    for (int j0 = 0; j0 < nb; j0 += 2) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            const int key = lane / PARTS + KPU * u, part = lane % PARTS;
            *reinterpret_cast<u32x4 *>(my + key * STRIDE + part * 16) = kreg[u];
        }
        __builtin_amdgcn_wave_barrier();

        f32x4 s[2], dp[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
            dp[h] = f32x4{0.f, 0.f, 0.f, 0.f};
            const char *krow = my + (h * 16 + i16) * STRIDE + g * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s[h] = mfma16(*reinterpret_cast<const bf16x8 *>(krow + ks * 64), qop[ks], s[h]);
                dp[h] = mfma16(vop[h][ks], gop[ks], dp[h]);
            }
        }
        const float c2[2] = {bias2[0] - lse2, bias2[1] - lse2};
        const int c[2] = {cnt[0], cnt[1]};
        if (j0 + 2 < nb) load_tile(j0 + 2);        // the K tile in LDS stays valid until the next iteration's stores

#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[h][r], sc2, c2[h]));
                s[h][r] = p * (dp[h][r] - delta);
            }
        if (c[0] < 16 || c[1] < 16) {              // ragged or absent block: its rows contribute nothing
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (4 * g + r >= c[h]) s[h][r] = 0.f;
        }
        const bf16x8 dsop = pack8(s[0], s[1]);
        const char *base = my + (4 * g + (i16 >> 2)) * STRIDE + (i16 & 3) * 8;
#pragma unroll
        for (int n = 0; n < NT; ++n)
            acc[n] = mfma16(lds_tr_pair(base + n * 32, base + 16 * STRIDE + n * 32), dsop, acc[n]);
    }

    uint16_t *orow = dQ + qrow * D + 4 * g;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        u32x2 w;
        w[0] = pack_bf16(acc[n][0] * t.scale, acc[n][1] * t.scale);
        w[1] = pack_bf16(acc[n][2] * t.scale, acc[n][3] * t.scale);
        *reinterpret_cast<u32x2 *>(orow + n * 16) = w;
    }
}

hipError_t launch_dq_mfma(const Plan &p, const LevelTable &t, const void *Q, const void *O, const void *dO,
                          const float *LSE, float *D, void *dQ, hipStream_t s) {
    if (p.N % 256 == 0 && (p.Kl[0] << (p.lb - 4)) <= 64) return launch_dq_shared(p, t, Q, O, dO, LSE, D, dQ, s);
    const int64_t wgs = (int64_t)p.bh * (p.N / 64);
    dim3 grid((unsigned)wgs);
    if (p.d == 64)
        dq_mfma_kernel<64><<<grid, 256, 0, s>>>(t, (const uint16_t *)Q, (const uint16_t *)O, (const uint16_t *)dO, LSE, D,
                                                (uint16_t *)dQ, p.N, wgs);
    else
        dq_mfma_kernel<128><<<grid, 256, 0, s>>>(t, (const uint16_t *)Q, (const uint16_t *)O, (const uint16_t *)dO, LSE,
                                                 D, (uint16_t *)dQ, p.N, wgs);
    return hipGetLastError();
}

}  // namespace llsa
