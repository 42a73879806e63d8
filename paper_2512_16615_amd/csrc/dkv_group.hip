// dK, dV of the coarse levels (l >= 1) on bf16 MFMA, grouped by query block (B = 16, d = 64, N % 256 == 0).
//
// The 256 fine queries under one level-1 query block R attend to the same coarse key blocks (Alg. 1,
// enrichment loop: fine block i reads row i / B^l of I^(l)).  Key-major processing (Sec. 4.3) re-reads the
// Q / dO rows of R once per listed key block; here one workgroup stages them once in LDS and each of its
// 8 waves takes some of R's coarse key blocks and runs the key-major tile loop over the 8 query tiles:
//   S = Q K^T, dP = dO V^T (lane: 4 queries x 1 key) -> P, dS -> dV^T += dO^T P, dK^T += Q^T dS.
// That yields, per (R, coarse block of R's list), the block's gradient restricted to R's queries: an 8 KB
// fp32 partial.  The partials are then added up in a fixed order:
//   1. levels l >= 2: the 16^(l-1) level-1 blocks under one level-l query block list the same key blocks,
//      so their partials are summed 16 at a time (slab_reduce16_kernel) until one partial per level-l
//      query block is left; the coarsest enriched level (every query attends to it) is summed down to one
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
    int64_t lvl_off[kMaxL + 1];                         // float offset of level l's partials [R][pos][kUnit]
    int nblk[kMaxL + 1];                                // key blocks of level l in a list
    int64_t N, NR;                                      // NR = level-1 query blocks per head
    int lev_end;                                        // levels 1 .. lev_end - 1 are processed here
    float sc2, scale;
};

__device__ __forceinline__ int swz(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }

__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4)))
dkv_group_kernel(LevelTable t, GroupArgs a) {
    constexpr int D = 64, KS = 2, NT = 4;
    __shared__ __attribute__((aligned(16))) char qs[256 * 128];       // Q rows of the group, chunk-swizzled
    __shared__ __attribute__((aligned(16))) char gs[256 * 128];       // dO rows
    __shared__ __attribute__((aligned(16))) float st[512];            // LSE | D

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i16 = lane & 15, g = lane >> 4;
    const int64_t R = xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t bh = R / a.NR, Rh = R % a.NR;
    const int64_t row0 = bh * a.N + Rh * 256;

    // ---- stage the group's Q, dO rows and statistics
    {
        const char *qsrc = reinterpret_cast<const char *>(a.Q + row0 * D), *gsrc = reinterpret_cast<const char *>(a.dO + row0 * D);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int cc = tid + 512 * k, r = cc >> 3, c = cc & 7;
            *reinterpret_cast<u32x4 *>(qs + swz(r, c)) = *reinterpret_cast<const u32x4 *>(qsrc + cc * 16);
            *reinterpret_cast<u32x4 *>(gs + swz(r, c)) = *reinterpret_cast<const u32x4 *>(gsrc + cc * 16);
        }
        st[tid] = tid < 256 ? a.LSE[row0 + tid] : a.Dsum[row0 + tid - 256];
    }
    __syncthreads();

    // per-lane LDS offsets (the swizzle key of a row depends only on the lane, see swz)
    const int key_row = (i16 >> 1) & 7, key_tr = (2 * g + (i16 >> 3)) & 7;
    int rowoff[KS], troff[NT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) rowoff[ks] = i16 * 128 + (((g + 4 * ks) ^ key_row) << 4);
#pragma unroll
    for (int n = 0; n < NT; ++n)
        troff[n] = (4 * g + (i16 >> 2)) * 128 + (((2 * n + ((i16 >> 1) & 1)) ^ key_tr) << 4) + ((i16 & 1) << 3);

    const int nlev = min(t.nlev, a.lev_end);
    const int c_begin = t.bseg[1], nbc = pick(t.bseg, nlev) - c_begin;
    BlockTable ctab;
    int chunk = -1;
    for (int jb = wave; jb < nbc; jb += 8) {
        if ((jb >> 6) != chunk) { chunk = jb >> 6; ctab.fill(t, bh, Rh * 16, c_begin, chunk, lane, D, nlev); }
        const char *kp = ctab.K(jb & 63), *vp = ctab.V(jb & 63);
        const int cnt = ctab.count(jb & 63);
        const float bias2 = ctab.bias(jb & 63);
        bf16x8 kop[KS], vop[KS];
        {
            const int off = (min(i16, cnt - 1) * D + g * 8) * 2;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                kop[ks] = ld_bf16x8(kp + off + 64 * ks);
                vop[ks] = ld_bf16x8(vp + off + 64 * ks);
            }
        }
        f32x4 accK[NT], accV[NT];
#pragma unroll
        for (int n = 0; n < NT; ++n) { accK[n] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[n] = f32x4{0.f, 0.f, 0.f, 0.f}; }

        for (int u = 0; u < 8; ++u) {                       // 8 tiles of 32 queries
            f32x4 s[2], dp[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int base = (32 * u + 16 * h) * 128;
                s[h] = f32x4{0.f, 0.f, 0.f, 0.f};
                dp[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    s[h] = mfma16(*reinterpret_cast<const bf16x8 *>(qs + base + rowoff[ks]), kop[ks], s[h]);
                    dp[h] = mfma16(*reinterpret_cast<const bf16x8 *>(gs + base + rowoff[ks]), vop[ks], dp[h]);
                }
                const f32x4 l2 = *reinterpret_cast<const f32x4 *>(st + 32 * u + 16 * h + 4 * g);
                const f32x4 dl = *reinterpret_cast<const f32x4 *>(st + 256 + 32 * u + 16 * h + 4 * g);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(s[h][r], a.sc2, fmaf(l2[r], -kLog2e, bias2)));
                    s[h][r] = p;
                    dp[h][r] = p * (dp[h][r] - dl[r]);
                }
            }
            const bf16x8 pop = pack8(s[0], s[1]), dsop = pack8(dp[0], dp[1]);
            const int b0 = 32 * u * 128, b1 = b0 + 16 * 128;
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                accV[n] = mfma16(lds_tr_pair(gs + b0 + troff[n], gs + b1 + troff[n]), pop, accV[n]);
                accK[n] = mfma16(lds_tr_pair(qs + b0 + troff[n], qs + b1 + troff[n]), dsop, accK[n]);
            }
        }

        // which level / position of R's list is block jb?  (wave-uniform)
        const int jl = jb + c_begin;
        int l = 1;
#pragma unroll
        for (int x = 2; x <= kMaxL; ++x) l += (x < nlev && jl >= t.bseg[x]) ? 1 : 0;
        const int pos = jl - pick(t.bseg, l);
        float *dst = a.slab + pick(a.lvl_off, l) + ((int64_t)R * pick(a.nblk, l) + pos) * kUnit + i16 * D + 4 * g;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            f32x4 k = accK[n];
#pragma unroll
            for (int r = 0; r < 4; ++r) k[r] *= a.scale;
            *reinterpret_cast<f32x4 *>(dst + n * 16) = k;
            *reinterpret_cast<f32x4 *>(dst + 16 * D + n * 16) = accV[n];
        }
    }
}

// out[h][r][x] = sum_{c < 16, 16 r + c < cnt_in} in[h][16 r + c][x], x over `width` floats (one thread per float4)
__global__ void __launch_bounds__(256) slab_reduce16_kernel(const float *in, float *out, int64_t cnt_in, int64_t cnt_out,
                                                             int64_t width4, int64_t total4) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total4) return;
    const int64_t x = i % width4, hr = i / width4, r = hr % cnt_out, h = hr / cnt_out;
    const int64_t first = 16 * r, n = min((int64_t)16, cnt_in - first);
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

// Highest level the grouped kernel takes; levels above it go to the split key-major kernel.  Only a wide dense
// coarsest level is left out: every query block would write a partial sum for every one of its key blocks, and
// summing over all queries is what the split kernel does in registers.  (Sending a coarsest level of a single
// key block to the split kernel, to spare the 8 waves a third round for one block, was measured slower.)
int dkv_group_top(const Plan &p) {
    if (p.Le == p.L && (p.n[p.L] + 15) / 16 > 32) return p.L - 1;
    return p.Le;
}

// bytes of the partial slab and of each of the two reduction buffers
void dkv_group_sizes(const Plan &p, size_t *slab_bytes, size_t *red_bytes) {
    const int64_t NR = p.N / 256;
    size_t slab = 0, red = 0;
    for (int l = 1; l <= dkv_group_top(p); ++l) {
        const int64_t nblk = l < p.L ? p.Kl[l] : (p.n[l] + 15) / 16;
        const size_t lv = (size_t)p.bh * NR * nblk * kUnit * sizeof(float);
        slab += lv;
        const size_t r = (size_t)p.bh * ((NR + 15) / 16) * nblk * kUnit * sizeof(float);
        if ((l >= 2 || l == p.L) && r > red) red = r;       // levels that get reduced before the gather
    }
    *slab_bytes = slab;
    *red_bytes = red;
}

hipError_t launch_dkv_group(const Plan &p, const LevelTable &t, const void *Q, const void *dO, const float *LSE,
                            const float *D, void *ws, hipStream_t s) {
    char *w = static_cast<char *>(ws);
    const int64_t NR = p.N / 256;
    GroupArgs a;
    a.Q = (const uint16_t *)Q; a.dO = (const uint16_t *)dO; a.LSE = LSE; a.Dsum = D;
    a.slab = (float *)(w + p.grp_slab_off);
    a.N = p.N; a.NR = NR;
    a.sc2 = p.scale * kLog2e; a.scale = p.scale;
    int64_t off = 0;
    const int top = dkv_group_top(p);
    a.lev_end = top + 1;
    for (int l = 0; l <= kMaxL; ++l) { a.lvl_off[l] = 0; a.nblk[l] = 0; }
    for (int l = 1; l <= top; ++l) {
        a.nblk[l] = l < p.L ? p.Kl[l] : (int)((p.n[l] + 15) / 16);
        a.lvl_off[l] = off;
        off += (int64_t)p.bh * NR * a.nblk[l] * kUnit;
    }
    dkv_group_kernel<<<dim3((unsigned)(p.bh * NR)), 512, 0, s>>>(t, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    float *red[2] = {(float *)(w + p.grp_red_off[0]), (float *)(w + p.grp_red_off[1])};
    for (int l = top; l >= 1; --l) {                        // top-down: a level adds the share of the one above
        const bool dense = (l == p.L);
        const float *cur = a.slab + a.lvl_off[l];
        int64_t cnt = NR;
        const int64_t target = dense ? 1 : p.n[l + 1];      // listers per head: level-l query blocks, or the head
        const int64_t width4 = (int64_t)a.nblk[l] * (kUnit / 4);
        int flip = 0;
        while (cnt > target) {
            const int64_t cnt_out = (cnt + 15) / 16;
            const int64_t total4 = (int64_t)p.bh * cnt_out * width4;
            slab_reduce16_kernel<<<dim3((unsigned)((total4 + 255) / 256)), 256, 0, s>>>(cur, red[flip], cnt, cnt_out, width4,
                                                                                        total4);
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
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace llsa
