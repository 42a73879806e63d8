// Attention forward over the gathered lists on bf16 MFMA (B = 16, d = 64 or 128): Alg. 1's attention loop
// with Eq. 1-5 evaluated tile by tile with an online softmax.
//
// One wave owns one fine query block (16 queries).  Per tile of two 16-token key blocks it computes
//   S^T = K Q^T   (A = key rows straight from global memory, B = the query block held in registers),
// so every lane ends up with 4 keys x 1 query of S^T; the softmax statistics of a query are then a
// reduction inside the lane plus two cross-lane steps, and the probabilities already sit in the register
// layout the second product wants as its B operand:
//   O^T += V^T P^T (A = V^T read from LDS with the transposing 64-bit read, B = P^T).
// V tiles are staged per wave in LDS (row-major, padded rows) because the second product contracts over
// keys while V is stored with d contiguous.
#include "mfma_common.h"

namespace llsa {

template <int D>
__global__ void __launch_bounds__(256) attn_fwd_mfma_kernel(LevelTable t, const uint16_t *__restrict__ Q,
                                                             uint16_t *__restrict__ O, float *__restrict__ LSE,
                                                             int64_t N, int64_t total_blocks) {
    constexpr int KS = D / 32;            // MFMA steps over d for S^T
    constexpr int NT = D / 16;            // 16-wide d tiles of O^T
    constexpr int STRIDE = D * 2 + 32;    // bytes per key row in LDS (padding spreads the rows over the banks)
    constexpr int VCH = D / 16;           // 16-byte chunks of a 32-key V tile per lane
    constexpr int PARTS = D / 8;          // 16-byte chunks per key row
    constexpr int KPU = 64 / PARTS;       // key rows covered by one chunk round of the wave
    __shared__ __attribute__((aligned(16))) char vlds[4][32 * STRIDE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t fb = (int64_t)blockIdx.x * 4 + wave;
    if (fb >= total_blocks) return;       // no workgroup barrier below: waves are independent
    const int64_t nblk = N >> 4, bh = fb / nblk, blk = fb % nblk;
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
    float m = -INFINITY, lsum = 0.f;
    const float sc2 = t.scale * 1.4426950408889634f;

    BlockWalker walk(t, bh, blk);
    KeyBlock kb[2];
    bf16x8 kop[2][KS];
    u32x4 vreg[VCH];

    auto load_tile = [&]() {
        kb[0] = walk.next(D);
        kb[1] = walk.next(D);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const KeyBlock &b = kb[h].cnt > 0 ? kb[h] : kb[0];       // an absent half re-reads valid memory
            const uint16_t *kr = b.K + min(i16, b.cnt - 1) * D + g * 8;
#pragma unroll
            for (int s = 0; s < KS; ++s) kop[h][s] = ld_bf16x8(kr + 32 * s);
        }
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            const int key = lane / PARTS + KPU * u, part = lane % PARTS, h = (KPU * u) >> 4;  // h is fixed per u
            const KeyBlock &b = kb[h].cnt > 0 ? kb[h] : kb[0];
            vreg[u] = *reinterpret_cast<const u32x4 *>(b.V + min(key & 15, b.cnt - 1) * D + part * 8);
        }
    };

    load_tile();
    while (true) {
        // stage this tile's V rows; LDS operations of one wave complete in order, the barrier only pins
        // the compiler's schedule
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < VCH; ++u) {
            const int key = lane / PARTS + KPU * u, part = lane % PARTS;
            *reinterpret_cast<u32x4 *>(my + key * STRIDE + part * 16) = vreg[u];
        }
        __builtin_amdgcn_wave_barrier();

        // S^T for both halves
        f32x4 s[2];
        float bias2[2];
        int cnt[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) s[h] = mfma16(kop[h][ks], qop[ks], s[h]);
            bias2[h] = kb[h].bias2;
            cnt[h] = kb[h].cnt;
        }
        const bool more = !walk.done();
        if (more) load_tile();                                       // next tile's loads fly during the math

        float mx = -INFINITY;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float z = (4 * g + r < cnt[h]) ? fmaf(s[h][r], sc2, bias2[h]) : -INFINITY;
                s[h][r] = z;
                mx = fmaxf(mx, z);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        float ps = 0.f;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = __builtin_amdgcn_exp2f(s[h][r] - m_new);
                s[h][r] = p;
                ps += p;
            }
        ps += __shfl_xor(ps, 16, 64);
        ps += __shfl_xor(ps, 32, 64);
        lsum = lsum * alpha + ps;
        m = m_new;
        const bf16x8 pop = pack8(s[0], s[1]);

        const char *base = my + (4 * g + (i16 >> 2)) * STRIDE + (i16 & 3) * 8;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const bf16x8 vop = lds_tr_pair(base + n * 32, base + 16 * STRIDE + n * 32);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[n][r] *= alpha;
            acc[n] = mfma16(vop, pop, acc[n]);
        }
        if (!more) break;
    }

    const float inv = 1.f / lsum;
    uint16_t *orow = O + (bh * N + blk * 16 + i16) * D + 4 * g;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        uint2 w;
        w.x = pack_bf16(acc[n][0] * inv, acc[n][1] * inv);
        w.y = pack_bf16(acc[n][2] * inv, acc[n][3] * inv);
        *reinterpret_cast<uint2 *>(orow + n * 16) = w;
    }
    if (g == 0) LSE[bh * N + blk * 16 + i16] = (m + __builtin_amdgcn_logf(lsum)) * 0.6931471805599453f;
}

hipError_t launch_attn_fwd_mfma(const Plan &p, const LevelTable &t, const void *Q, void *O, float *LSE,
                                hipStream_t s) {
    const int64_t total = (int64_t)p.bh * (p.N / 16);
    dim3 grid((unsigned)((total + 3) / 4));
    if (p.d == 64)
        attn_fwd_mfma_kernel<64><<<grid, 256, 0, s>>>(t, (const uint16_t *)Q, (uint16_t *)O, LSE, p.N, total);
    else
        attn_fwd_mfma_kernel<128><<<grid, 256, 0, s>>>(t, (const uint16_t *)Q, (uint16_t *)O, LSE, p.N, total);
    return hipGetLastError();
}

}  // namespace llsa
