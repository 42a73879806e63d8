// Portable scalar (VALU) kernels for every step of the LLSA layer, any supported shape and both I/O
// types.  The pooling, selection, index-transpose, D = rowsum(dO*O) and un-pooling kernels here are the
// ones every configuration uses; the attention / dQ / dK,dV kernels here are the fallback (and the fp32
// path), the bf16 B=16 shapes normally run the MFMA kernels instead.
#include "llsa_internal.h"

#include <math.h>

namespace llsa {

// ------------------------------------------------------------------------------------------ element types
struct bf16_t { uint16_t v; };

__device__ __forceinline__ float to_f(float x) { return x; }
__device__ __forceinline__ float to_f(bf16_t x) { return __uint_as_float(((uint32_t)x.v) << 16); }

template <class T> __device__ __forceinline__ T from_f(float f);
template <> __device__ __forceinline__ float from_f<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float f) {
    // round to nearest even; inf / nan pass through unchanged in their upper half
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) != 0x7f800000u) u += 0x7fffu + ((u >> 16) & 1u);
    bf16_t r; r.v = (uint16_t)(u >> 16);
    return r;
}

template <class T> struct Vec;                       // 16-byte vector of T
template <> struct Vec<float>  { static constexpr int n = 4; };
template <> struct Vec<bf16_t> { static constexpr int n = 8; };

template <class T> __device__ __forceinline__ void load_vec(const T *p, float *out);
template <> __device__ __forceinline__ void load_vec<float>(const float *p, float *out) {
    float4 v = *reinterpret_cast<const float4 *>(p);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
template <> __device__ __forceinline__ void load_vec<bf16_t>(const bf16_t *p, float *out) {
    uint4 v = *reinterpret_cast<const uint4 *>(p);
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(w[i] << 16);
        out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
template <class T> __device__ __forceinline__ void store_vec(T *p, const float *in);
template <> __device__ __forceinline__ void store_vec<float>(float *p, const float *in) {
    *reinterpret_cast<float4 *>(p) = make_float4(in[0], in[1], in[2], in[3]);
}
template <> __device__ __forceinline__ void store_vec<bf16_t>(bf16_t *p, const float *in) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        w[i] = (uint32_t)from_f<bf16_t>(in[2 * i]).v | ((uint32_t)from_f<bf16_t>(in[2 * i + 1]).v << 16);
    *reinterpret_cast<uint4 *>(p) = make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// plain fp32 dot of a row in global memory with a vector held in LDS (fp32)
template <class T> __device__ __forceinline__ float dot_row(const T *row, const float *x, int d) {
    float s = 0.f, tmp[Vec<T>::n];
    for (int c = 0; c < d; c += Vec<T>::n) {
        load_vec<T>(row + c, tmp);
#pragma unroll
        for (int e = 0; e < Vec<T>::n; ++e) s = fmaf(tmp[e], x[c + e], s);
    }
    return s;
}

// ------------------------------------------------------------------------------------------------ pooling
// Alg. 1, compression loop: out[t] = (x[tB] + x[tB+1] + ... + x[tB+B-1]) / B, summed in that order in
// fp32, one IEEE division, one rounding to the I/O type.  The order is part of the contract: the
// selection below is decided on these values, so they must not depend on the launch shape.
struct PoolArgs { const void *in[3]; void *out[3]; void *out2[3]; };

// BC: block size known at compile time (the row loop is unrolled, so all B loads of a thread are in flight at once),
// or 0 to take it from the argument.  Same order of additions either way.
// TWO: the workgroup also pools its own output once more (out2 = the level above): its 256 / (d / VN) output tokens
// are whole groups of B, their rounded values pass through LDS and are summed in the same ascending order, so out2
// is bit for bit what a second launch on `out` would write, without that launch.
template <class T, int BC, bool TWO>
__global__ void __launch_bounds__(256) pool_kernel(PoolArgs a, int64_t n_out_total, int d, int B_arg) {
    constexpr int VN = Vec<T>::n;
    __shared__ float lvl[TWO ? 256 * VN : 1];
    const int B = BC ? BC : B_arg;
    const int vpr = d / VN;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t t = idx / vpr;
    const int cv = (int)(idx % vpr);
    const bool live = t < n_out_total;
    if (!TWO && !live) return;
    float s[VN];
#pragma unroll
    for (int e = 0; e < VN; ++e) s[e] = 0.f;
    if (live) {
        const T *in = static_cast<const T *>(a.in[blockIdx.y]) + (t * B) * (int64_t)d + cv * VN;
        if constexpr (BC != 0) {
            float x[BC][VN];
#pragma unroll
            for (int r = 0; r < BC; ++r) load_vec<T>(in + (int64_t)r * d, x[r]);
#pragma unroll
            for (int r = 0; r < BC; ++r)
#pragma unroll
                for (int e = 0; e < VN; ++e) s[e] = s[e] + x[r][e];
        } else {
            int r0 = 0;
            for (; r0 + 16 <= B; r0 += 16) {                   // 16 rows in flight at a time, added in row order
                float x[16][VN];
#pragma unroll
                for (int r = 0; r < 16; ++r) load_vec<T>(in + (int64_t)(r0 + r) * d, x[r]);
#pragma unroll
                for (int r = 0; r < 16; ++r)
#pragma unroll
                    for (int e = 0; e < VN; ++e) s[e] = s[e] + x[r][e];
            }
            float x[VN];
            for (int r = r0; r < B; ++r) {
                load_vec<T>(in + (int64_t)r * d, x);
#pragma unroll
                for (int e = 0; e < VN; ++e) s[e] = s[e] + x[e];
            }
        }
        const float Bf = (float)B;
#pragma unroll
        for (int e = 0; e < VN; ++e) s[e] = __fdiv_rn(s[e], Bf);
        store_vec<T>(static_cast<T *>(a.out[blockIdx.y]) + t * (int64_t)d + cv * VN, s);
    }
    if constexpr (TWO) {
#pragma unroll
        for (int e = 0; e < VN; ++e) lvl[threadIdx.x * VN + e] = to_f(from_f<T>(s[e]));   // what was stored, as fp32
        __syncthreads();
        const int tpw = 256 / vpr;                         // output tokens of this workgroup: tpw / B whole groups
        const int t2l = threadIdx.x / vpr;                 // group this thread sums (threads beyond the groups idle)
        const int64_t first = (int64_t)blockIdx.x * tpw;   // the workgroup's first output token: a multiple of B
        if (t2l < tpw / B && first + (int64_t)(t2l + 1) * B <= n_out_total) {
            float u[VN];
#pragma unroll
            for (int e = 0; e < VN; ++e) u[e] = 0.f;
            for (int r = 0; r < B; ++r)
#pragma unroll
                for (int e = 0; e < VN; ++e) u[e] = u[e] + lvl[((t2l * B + r) * vpr + cv) * VN + e];
            const float Bf = (float)B;
#pragma unroll
            for (int e = 0; e < VN; ++e) u[e] = __fdiv_rn(u[e], Bf);
            store_vec<T>(static_cast<T *>(a.out2[blockIdx.y]) + (first / B + t2l) * (int64_t)d + cv * VN, u);
        }
    }
}

hipError_t launch_pool(const Plan &p, const void *Q, const void *K, const void *V, void *ws, bool q_too,
                       hipStream_t s) {
    const void *src[3] = {Q, K, V};
    char *w = static_cast<char *>(ws);
    const int vn = 16 / p.elt;
    // levels 1 and 2 in one launch where a workgroup's 256 / (d / vn) level-1 tokens are whole groups of B
    const bool two = p.L >= 2 && p.elt == 2 && p.B == 16 && (256 / (p.d / vn)) % p.B == 0;
    for (int l = 1; l <= p.L; ++l) {
        if (two && l == 2) continue;
        PoolArgs a;
        int cnt = 0;
        for (int x = q_too ? 0 : 1; x < 3; ++x, ++cnt) {
            a.in[cnt] = (l == 1) ? src[x] : (const void *)(w + p.pyr_off[x][l - 1]);
            a.out[cnt] = w + p.pyr_off[x][l];
            a.out2[cnt] = (two && l == 1) ? (void *)(w + p.pyr_off[x][2]) : nullptr;
        }
        const int64_t n_out_total = (int64_t)p.bh * p.n[l];
        const int64_t threads = n_out_total * (p.d / vn);
        dim3 grid((unsigned)((threads + 255) / 256), cnt);
        if (p.elt == 4) pool_kernel<float, 0, false><<<grid, 256, 0, s>>>(a, n_out_total, p.d, p.B);
        else if (two && l == 1) pool_kernel<bf16_t, 16, true><<<grid, 256, 0, s>>>(a, n_out_total, p.d, p.B);
        else if (p.B == 16) pool_kernel<bf16_t, 16, false><<<grid, 256, 0, s>>>(a, n_out_total, p.d, p.B);
        else                pool_kernel<bf16_t, 0, false><<<grid, 256, 0, s>>>(a, n_out_total, p.d, p.B);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ----------------------------------------------------------------------- layer glue fused with pooling
// QK-Norm and RoPE in front of the layer (Sec. 5.2, "Training Settings") fused with the first step of the
// compression loop of Alg. 1: one pass over the pre-norm tensor writes the level-0 tensor the layer consumes
// and its level-1 mean, so the level-0 tensor is never read back for pooling.
//   y[c]      = x[c] / sqrt(mean_c(x^2) + eps) * gamma[c]                      (per token, over the head dimension)
//   out[2i]   = y[2i] cos[t][i] - y[2i+1] sin[t][i]
//   out[2i+1] = y[2i] sin[t][i] + y[2i+1] cos[t][i]                             (t: token index within the head)
// out is rounded to the I/O type; the level-1 token is pooled from those rounded values exactly as pool_kernel
// does it (ascending fp32 sum, one division, one rounding), so it equals pool_kernel's result on `out` bit for bit.
// One thread per (level-1 token, 16-byte channel vector); the d / VN threads of a token are neighbouring lanes and
// reduce the sum of squares of a row with xor shuffles.  grid.y: 0 = Q, 1 = K.
struct GlueArgs { const void *in[2]; void *out[2]; void *lvl1[2]; const float *gamma[2]; };

template <class T>
__global__ void __launch_bounds__(256) qknorm_rope_pool_kernel(GlueArgs a, const float *__restrict__ cos_t,
                                                               const float *__restrict__ sin_t, float eps,
                                                               int64_t n1_total, int64_t N, int d, int B) {
    constexpr int VN = Vec<T>::n, ROWS = 4;                // rows of one token group in flight at a time
    const int vpr = d / VN;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t t1 = idx / vpr;                          // level-1 token, flat over (batch, head)
    const int cv = (int)(idx % vpr);
    if (t1 >= n1_total) return;                            // whole token groups leave together (vpr divides 64)
    const int y = blockIdx.y;
    const T *in = static_cast<const T *>(a.in[y]) + (t1 * B) * (int64_t)d + cv * VN;
    T *out = static_cast<T *>(a.out[y]) + (t1 * B) * (int64_t)d + cv * VN;
    const int64_t tok0 = (t1 * B) % N;                     // position of the group's first token inside its head
    float gam[VN];
#pragma unroll
    for (int e = 0; e < VN; ++e) gam[e] = a.gamma[y][cv * VN + e];
    const float inv_d = 1.f / (float)d;
    float s[VN];
#pragma unroll
    for (int e = 0; e < VN; ++e) s[e] = 0.f;
    for (int r0 = 0; r0 < B; r0 += ROWS) {
        float x[ROWS][VN], cs[ROWS][VN / 2], sn[ROWS][VN / 2];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            const int rr = min(r0 + r, B - 1);             // B need not be a multiple of ROWS: the tail re-reads
            load_vec<T>(in + (int64_t)rr * d, x[r]);
            const int64_t tab = (tok0 + rr) * (d / 2) + cv * (VN / 2);
#pragma unroll
            for (int e = 0; e < VN / 2; ++e) { cs[r][e] = cos_t[tab + e]; sn[r][e] = sin_t[tab + e]; }
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            float ss = 0.f;
#pragma unroll
            for (int e = 0; e < VN; ++e) ss = fmaf(x[r][e], x[r][e], ss);
            for (int o = 1; o < vpr; o <<= 1) ss += __shfl_xor(ss, o, 64);
            const float rinv = 1.f / sqrtf(fmaf(ss, inv_d, eps));
            float o8[VN];
#pragma unroll
            for (int e = 0; e < VN / 2; ++e) {
                const float y0 = x[r][2 * e] * rinv * gam[2 * e], y1 = x[r][2 * e + 1] * rinv * gam[2 * e + 1];
                o8[2 * e] = to_f(from_f<T>(y0 * cs[r][e] - y1 * sn[r][e]));
                o8[2 * e + 1] = to_f(from_f<T>(y0 * sn[r][e] + y1 * cs[r][e]));
            }
            if (r0 + r < B) {
                store_vec<T>(out + (int64_t)(r0 + r) * d, o8);
#pragma unroll
                for (int e = 0; e < VN; ++e) s[e] = s[e] + o8[e];
            }
        }
    }
    const float Bf = (float)B;
#pragma unroll
    for (int e = 0; e < VN; ++e) s[e] = __fdiv_rn(s[e], Bf);
    store_vec<T>(static_cast<T *>(a.lvl1[y]) + t1 * (int64_t)d + cv * VN, s);
}

// Q and K through the fused kernel, V's level 1 and every level above through pool_kernel.
hipError_t launch_qknorm_rope_pool(const Plan &p, const void *Qpre, const void *Kpre, const void *V,
                                   const float *gamma_q, const float *gamma_k, const float *cos_t, const float *sin_t,
                                   float eps, void *Qout, void *Kout, void *ws, hipStream_t s) {
    char *w = static_cast<char *>(ws);
    GlueArgs g;
    g.in[0] = Qpre; g.in[1] = Kpre;
    g.out[0] = Qout; g.out[1] = Kout;
    g.lvl1[0] = w + p.pyr_off[0][1]; g.lvl1[1] = w + p.pyr_off[1][1];
    g.gamma[0] = gamma_q; g.gamma[1] = gamma_k;
    const int vn = 16 / p.elt;
    const int64_t n1_total = (int64_t)p.bh * p.n[1];
    const int64_t threads = n1_total * (p.d / vn);
    dim3 grid((unsigned)((threads + 255) / 256), 2);
    if (p.elt == 4) qknorm_rope_pool_kernel<float><<<grid, 256, 0, s>>>(g, cos_t, sin_t, eps, n1_total, p.N, p.d, p.B);
    else qknorm_rope_pool_kernel<bf16_t><<<grid, 256, 0, s>>>(g, cos_t, sin_t, eps, n1_total, p.N, p.d, p.B);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const void *src[3] = {Qout, Kout, V};
    for (int l = 1; l <= p.L; ++l) {
        PoolArgs a;
        int cnt = 0;
        for (int x = (l == 1) ? 2 : 0; x < 3; ++x, ++cnt) {    // level 1 of Q and K is already there
            a.in[cnt] = (l == 1) ? src[x] : (const void *)(w + p.pyr_off[x][l - 1]);
            a.out[cnt] = w + p.pyr_off[x][l];
            a.out2[cnt] = nullptr;
        }
        const int64_t n_out_total = (int64_t)p.bh * p.n[l];
        const int64_t th = n_out_total * (p.d / vn);
        dim3 pg((unsigned)((th + 255) / 256), cnt);
        if (p.elt == 4) pool_kernel<float, 0, false><<<pg, 256, 0, s>>>(a, n_out_total, p.d, p.B);
        else if (p.B == 16) pool_kernel<bf16_t, 16, false><<<pg, 256, 0, s>>>(a, n_out_total, p.d, p.B);
        else                pool_kernel<bf16_t, 0, false><<<pg, 256, 0, s>>>(a, n_out_total, p.d, p.B);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------------------------- selection
// Alg. 1, selection loop, one level: every wave scores one level-l query token against its candidates
// (all n_L tokens at the coarsest level, the K_l*B children of the parent's picks below it) and keeps the
// Kout best.  Scores are fp32 fused-multiply-add chains over channels 0..d-1 in order, so they do not
// depend on the launch shape; ties go to the lower key id; rows are written in ascending id order.
template <class T>
__global__ void select_kernel(const T *Ql, const T *Kl, int64_t n_l, int d, int B, const int32_t *parent, int Kp,
                              int Kout, int32_t *out, int C, int64_t nblk) {
    extern __shared__ float smem[];
    const int W = blockDim.x >> 6, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float *qs = smem + wave * d;
    float *sc = smem + W * d + (size_t)wave * C;
    const int64_t bh = blockIdx.x / nblk, r = blockIdx.x % nblk;
    const T *Kb = Kl + bh * n_l * d;
    const int32_t *prow = parent ? parent + (bh * nblk + r) * Kp : nullptr;
    const int iters = (B + W - 1) / W;
    for (int it = 0; it < iters; ++it) {
        const int u = it * W + wave;
        const int64_t i = r * B + u;
        const bool active = (u < B) && (i < n_l);
        __syncthreads();                                   // previous row's LDS no longer read
        if (active)
            for (int c = lane; c < d; c += 64) qs[c] = to_f(Ql[(bh * n_l + i) * d + c]);
        __syncthreads();
        if (active)
            for (int p = lane; p < C; p += 64) {
                const int64_t id = prow ? (int64_t)prow[p / B] * B + p % B : p;
                const T *k = Kb + id * d;
                float s = 0.f, tmp[Vec<T>::n];
                for (int c = 0; c < d; c += Vec<T>::n) {
                    load_vec<T>(k + c, tmp);
#pragma unroll
                    for (int e = 0; e < Vec<T>::n; ++e) s = __builtin_fmaf(qs[c + e], tmp[e], s);
                }
                sc[p] = s;
            }
        int mine = 0;                                      // lane k keeps the k-th winner's position
        for (int k = 0; k < Kout; ++k) {
            __syncthreads();
            float bs = -INFINITY;
            int bp = 0x7fffffff;
            if (active)
                for (int p = lane; p < C; p += 64) {
                    const float v = sc[p];
                    if (v > bs) { bs = v; bp = p; }        // ascending p: strict '>' keeps the lowest position
                }
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) {
                const float os = __shfl_xor(bs, o, 64);
                const int op = __shfl_xor(bp, o, 64);
                if (os > bs || (os == bs && op < bp)) { bs = os; bp = op; }
            }
            if (active && lane == (bp & 63)) sc[bp] = -INFINITY;
            if (lane == k) mine = bp;
        }
        if (active) {
            // candidate positions ascend with key id (parent rows are ascending), so rank by position
            int rank = 0;
            for (int k = 0; k < Kout; ++k) rank += (__shfl(mine, k, 64) < mine) ? 1 : 0;
            if (lane < Kout) {
                const int64_t id = prow ? (int64_t)prow[mine / B] * B + mine % B : mine;
                out[(bh * n_l + i) * Kout + rank] = (int32_t)id;
            }
        }
    }
}

hipError_t launch_select(const Plan &p, int l, const void *ws, const int32_t *parent, int32_t *out, hipStream_t s) {
    if (p.desc.kernel_path == 0 && select_fast_ok(p, l)) return launch_select_fast(p, l, ws, parent, out, s);
    const char *w = static_cast<const char *>(ws);
    const bool top = (l == p.L);
    const int C = top ? (int)p.n[l] : p.Kl[l] * p.B;
    const int Kout = p.Kl[l - 1];
    const int64_t nblk = (p.n[l] + p.B - 1) / p.B;
    const int W = C <= 2048 ? 4 : (C <= 4096 ? 2 : 1);
    const size_t lds = (size_t)W * (p.d + C) * sizeof(float);
    dim3 grid((unsigned)(p.bh * nblk));
    const int Kp = top ? 0 : p.Kl[l];
    const void *Ql = w + p.pyr_off[0][l], *Kl = w + p.pyr_off[1][l];
    if (p.elt == 4)
        select_kernel<float><<<grid, W * 64, lds, s>>>((const float *)Ql, (const float *)Kl, p.n[l], p.d, p.B,
                                                       top ? nullptr : parent, Kp, Kout, out, C, nblk);
    else
        select_kernel<bf16_t><<<grid, W * 64, lds, s>>>((const bf16_t *)Ql, (const bf16_t *)Kl, p.n[l], p.d, p.B,
                                                        top ? nullptr : parent, Kp, Kout, out, C, nblk);
    return hipGetLastError();
}

// -------------------------------------------------------------------------------------- gathered-list walk
// Position `pos` of the list of fine query block `blk` (Alg. 1, enrichment loop): level and token id.
__device__ __forceinline__ void list_entry(const LevelTable &t, int64_t bh, int64_t blk, int pos, int &lev,
                                           int &tok) {
    int l = 0;
    while (l + 1 < t.nlev && pos >= t.seg[l + 1]) ++l;
    const int off = pos - t.seg[l];
    if (l < t.L) {
        const int64_t row = blk / t.Bpow[l];
        const int k = off / t.B, u = off % t.B;
        tok = t.I[l][(bh * t.rows[l] + row) * t.Kl[l] + k] * t.B + u;
    } else {
        tok = off;
    }
    lev = l;
}

// ------------------------------------------------------------------------------ attention forward (scalar)
// Eq. 1-5 restricted to the gathered list, one wave per query row, online softmax over chunks of 64 list
// entries (lane = entry for the logits, lane = channel for the value accumulation).
template <class T>
__global__ void __launch_bounds__(256) attn_fwd_generic(LevelTable t, const T *Q, T *O, float *LSE, int64_t N,
                                                         int64_t total_rows) {
    __shared__ float qs[4][128];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, d = t.d;
    int64_t row = (int64_t)blockIdx.x * 4 + wave;
    const bool active = row < total_rows;
    if (!active) row = total_rows - 1;
    const int64_t bh = row / N, q = row % N, blk = q / t.B;
    for (int c = lane; c < d; c += 64) qs[wave][c] = to_f(Q[row * d + c]);
    __syncthreads();
    const int M = t.seg[t.nlev];
    float m = -INFINITY, lsum = 0.f, acc0 = 0.f, acc1 = 0.f;
    for (int base = 0; base < M; base += 64) {
        const int pos = base + lane;
        const bool valid = pos < M;
        int lev = 0, tok = 0;
        float z = -INFINITY;
        if (valid) {
            list_entry(t, bh, blk, pos, lev, tok);
            const T *k = static_cast<const T *>(t.K[lev]) + (bh * t.n[lev] + tok) * d;
            z = t.scale * dot_row<T>(k, qs[wave], d) + t.bias[lev];
        }
        const float m_new = fmaxf(m, wave_max(z));
        const float pr = valid ? expf(z - m_new) : 0.f;
        const float alpha = expf(m - m_new);
        lsum = lsum * alpha + wave_sum(pr);
        acc0 *= alpha;
        acc1 *= alpha;
        m = m_new;
        const int cnt = min(64, M - base);
        for (int j = 0; j < cnt; ++j) {
            const float pj = __shfl(pr, j, 64);
            const int lj = __shfl(lev, j, 64), tj = __shfl(tok, j, 64);
            const T *v = static_cast<const T *>(t.V[lj]) + (bh * t.n[lj] + tj) * d;
            if (lane < d) acc0 = fmaf(pj, to_f(v[lane]), acc0);
            if (lane + 64 < d) acc1 = fmaf(pj, to_f(v[lane + 64]), acc1);
        }
    }
    if (active) {
        const float inv = 1.f / lsum;
        if (lane < d) O[row * d + lane] = from_f<T>(acc0 * inv);
        if (lane + 64 < d) O[row * d + lane + 64] = from_f<T>(acc1 * inv);
        if (lane == 0) LSE[row] = m + logf(lsum);
    }
}

hipError_t launch_attn_fwd_generic(const Plan &p, const LevelTable &t, const void *Q, void *O, float *LSE,
                                   hipStream_t s) {
    const int64_t rows = (int64_t)p.bh * p.N;
    dim3 grid((unsigned)((rows + 3) / 4));
    if (p.elt == 4) attn_fwd_generic<float><<<grid, 256, 0, s>>>(t, (const float *)Q, (float *)O, LSE, p.N, rows);
    else attn_fwd_generic<bf16_t><<<grid, 256, 0, s>>>(t, (const bf16_t *)Q, (bf16_t *)O, LSE, p.N, rows);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------- D = rowsum(dO * O)
template <class T>
__global__ void __launch_bounds__(256) bwd_pre_kernel(const T *O, const T *dO, float *D, int64_t rows, int d) {
    const int sub = threadIdx.x & 15;
    int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const bool active = row < rows;
    if (!active) row = rows - 1;
    float s = 0.f;
    for (int c = sub; c < d; c += 16) s = fmaf(to_f(O[row * d + c]), to_f(dO[row * d + c]), s);
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
    if (active && sub == 0) D[row] = s;
}

hipError_t launch_bwd_pre(const Plan &p, const void *O, const void *dO, float *D, hipStream_t s) {
    const int64_t rows = (int64_t)p.bh * p.N;
    dim3 grid((unsigned)((rows + 15) / 16));
    if (p.elt == 4) bwd_pre_kernel<float><<<grid, 256, 0, s>>>((const float *)O, (const float *)dO, D, rows, p.d);
    else bwd_pre_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)O, (const bf16_t *)dO, D, rows, p.d);
    return hipGetLastError();
}

// -------------------------------------------------------------------------------- index transpose (Alg. 2)
// count -> exclusive scan -> fill -> per-key ascending order.  Counting and filling use integer atomics;
// the order they leave inside a key's list depends on timing, so a last pass sorts every list (an entry counts the
// smaller ones of its list; lists of more than 4096 entries: a bitmap of the list's rows), which makes
// the result (and with it the summation order of dK / dV) the same on every run.
// All levels run in the same launches: blockIdx.y selects the level.
struct CscLevel {
    const int32_t *I;            // I^(l) [bh, T, Kl]
    int32_t *cnt, *C, *Iq, *Iq_tmp;
    int64_t T, eph, total, nk;   // keys per head, entries per head, entries, keys
    int Kl;
};
struct CscLevels { CscLevel lv[kMaxL]; };

__global__ void csc_zero_kernel(CscLevels a) {
    const CscLevel &L = a.lv[blockIdx.y];
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < L.nk) L.cnt[i] = 0;
}
__global__ void csc_count_kernel(CscLevels a) {
    const CscLevel &L = a.lv[blockIdx.y];
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= L.total) return;
    const int64_t bh = e / L.eph;
    atomicAdd(&L.cnt[bh * L.T + L.I[e]], 1);
}
// one workgroup per (head, level): C = exclusive scan of cnt (T+1 entries), cnt reset to 0 for the fill pass.
// 256 threads, so that a workgroup finds room on a CU beside the LDS-bound dK/dV kernels it runs in the shadow of
// (with 1024 threads it waited for a whole CU to drain).
constexpr int kScanThreads = 256;
__global__ void __launch_bounds__(kScanThreads) csc_scan_kernel(CscLevels a) {
    constexpr int NW = kScanThreads / 64;
    __shared__ int32_t wsum[NW];
    __shared__ int32_t carry;
    const CscLevel &L = a.lv[blockIdx.y];
    const int64_t bh = blockIdx.x, T = L.T;
    int32_t *cn = L.cnt + bh * T, *Co = L.C + bh * (T + 1);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < T; base += 4 * kScanThreads) {
        // four consecutive keys per thread
        const int64_t i0 = base + 4 * threadIdx.x;
        int32_t v[4], x = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[k] = i0 + k < T ? cn[i0 + k] : 0; x += v[k]; }
        const int32_t mine = x;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {                  // inclusive scan of the threads' sums inside the wave
            const int32_t y = __shfl_up(x, o, 64);
            if (lane >= o) x += y;
        }
        if (lane == 63) wsum[wave] = x;
        __syncthreads();
        int32_t pre = carry;
        for (int w2 = 0; w2 < wave; ++w2) pre += wsum[w2];
        int32_t run = pre + x - mine;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k < T) { Co[i0 + k] = run; cn[i0 + k] = 0; }
            run += v[k];
        }
        __syncthreads();
        if (threadIdx.x == kScanThreads - 1) carry = pre + x;
        __syncthreads();
    }
    if (threadIdx.x == 0) Co[T] = carry;
}
__global__ void csc_fill_kernel(CscLevels a) {
    const CscLevel &L = a.lv[blockIdx.y];
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= L.total) return;
    const int64_t bh = e / L.eph, within = e % L.eph;
    const int32_t key = L.I[e];
    const int32_t slot = L.C[bh * (L.T + 1) + key] + atomicAdd(&L.cnt[bh * L.T + key], 1);
    L.Iq_tmp[bh * L.eph + slot] = (int32_t)(within / L.Kl);
}
// one thread per list entry: its rank among the entries of the same key (entries are distinct query rows)
// is its place in the key's ascending list.  The unsorted list is re-read through the caches.
// Lists longer than kLongList are left to csc_sort_long_kernel (this pass costs len reads per entry).  A list is no
// longer than the level has rows, so levels of up to kLongList rows (the headline's level 0 has 4096) need no second pass.
constexpr int kLongList = 4096;
__global__ void __launch_bounds__(256) csc_sort_kernel(CscLevels a) {
    const CscLevel &L = a.lv[blockIdx.y];
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= L.total) return;
    const int64_t bh = e / L.eph, within = e % L.eph;
    const int32_t key = L.I[e], x = (int32_t)(within / L.Kl);
    const int32_t beg = L.C[bh * (L.T + 1) + key], end = L.C[bh * (L.T + 1) + key + 1];
    if (end - beg > kLongList) return;
    const int32_t *src = L.Iq_tmp + bh * L.eph;
    int32_t rank = 0;
    for (int32_t b = beg; b < end; ++b) rank += (src[b] < x) ? 1 : 0;
    L.Iq[bh * L.eph + beg + rank] = x;
}
// Long lists: every lane of a wave looks at one key, and the wave then works through the long lists among its 64
// keys together (usually none): the list's rows are marked in a bitmap of kSegRows rows at a time in LDS, and an
// entry's place is the number of marked rows below it: one pass over the list per segment of rows instead of one
// pass per entry, whatever the atomic fill's order was.  Keeps the transpose linear in the list length when many
// queries pick the same key (constant keys: every row lists blocks 0 .. K-1).
constexpr int kSegRows = 8192, kSegWords = kSegRows / 32;
__global__ void __launch_bounds__(256) csc_sort_long_kernel(CscLevels a) {
    __shared__ uint32_t bm_sh[4][kSegWords];
    __shared__ int32_t pre_sh[4][kSegWords];
    const CscLevel &L = a.lv[blockIdx.y];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t key0 = ((int64_t)blockIdx.x * 4 + wave) * 64;          // this wave's keys (over all heads)
    if (key0 >= L.nk) return;
    const int64_t mykey = min(key0 + lane, L.nk - 1);
    const int32_t mybeg = L.C[(mykey / L.T) * (L.T + 1) + mykey % L.T];
    const int32_t mylen = L.C[(mykey / L.T) * (L.T + 1) + mykey % L.T + 1] - mybeg;
    uint64_t todo = __ballot(key0 + lane < L.nk && mylen > kLongList);
    uint32_t *bm = bm_sh[wave];
    int32_t *pre = pre_sh[wave];
    while (todo) {
        const int j = (int)__builtin_ctzll(todo);
        todo &= todo - 1;
        const int64_t bh = (key0 + j) / L.T;
        const int32_t beg = __shfl(mybeg, j, 64), len = __shfl(mylen, j, 64);
        const int32_t *src = L.Iq_tmp + bh * L.eph + beg;
        int32_t *dst = L.Iq + bh * L.eph + beg;
        int32_t base = 0;                                   // entries in the segments done so far
        for (int64_t s0 = 0; s0 < L.T; s0 += kSegRows) {
            for (int w = lane; w < kSegWords; w += 64) bm[w] = 0u;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (int32_t e = lane; e < len; e += 64) {
                const int64_t x = src[e] - s0;
                if (x >= 0 && x < kSegRows) atomicOr(&bm[x >> 5], 1u << (x & 31));
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            // marked rows below every word: lane holds kSegWords / 64 consecutive words
            constexpr int PL = kSegWords / 64;
            int32_t c[PL], mine = 0;
#pragma unroll
            for (int i = 0; i < PL; ++i) { c[i] = __popc(bm[PL * lane + i]); mine += c[i]; }
            int32_t incl = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int32_t y = __shfl_up(incl, o, 64);
                if (lane >= o) incl += y;
            }
            int32_t run = incl - mine;
#pragma unroll
            for (int i = 0; i < PL; ++i) { pre[PL * lane + i] = run; run += c[i]; }
            const int32_t total = __shfl(incl, 63, 64);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
            for (int32_t e = lane; e < len; e += 64) {
                const int32_t v = src[e];
                const int64_t x = v - s0;
                if (x >= 0 && x < kSegRows) {
                    const int w = (int)(x >> 5);
                    dst[base + pre[w] + __popc(bm[w] & ((1u << (x & 31)) - 1u))] = v;
                }
            }
            base += total;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();                // the bitmap is cleared again only after these reads
        }
    }
}

// Alg. 2 for levels 0 .. top (the levels whose lists the backward uses), five launches in all (six for long levels)
hipError_t launch_csc(const Plan &p, int top, const int32_t *indices, void *ws, hipStream_t s) {
    char *w = static_cast<char *>(ws);
    CscLevels a;
    int64_t max_nk = 0, max_total = 0;
    for (int l = 0; l <= top; ++l) {
        CscLevel &L = a.lv[l];
        L.T = p.n[l + 1];
        L.Kl = p.Kl[l];
        L.eph = L.T * L.Kl;
        L.total = L.eph * p.bh;
        L.nk = L.T * p.bh;
        L.I = reinterpret_cast<const int32_t *>(reinterpret_cast<const char *>(indices) + p.idx_off[l]);
        L.cnt = (int32_t *)(w + p.cnt_off[l]);
        L.C = (int32_t *)(w + p.C_off[l]);
        L.Iq = (int32_t *)(w + p.Iq_off[l]);
        L.Iq_tmp = (int32_t *)(w + p.Iqtmp_off[l]);
        if (L.nk > max_nk) max_nk = L.nk;
        if (L.total > max_total) max_total = L.total;
    }
    const unsigned nl = (unsigned)(top + 1);
    csc_zero_kernel<<<dim3((unsigned)((max_nk + 255) / 256), nl), 256, 0, s>>>(a);
    csc_count_kernel<<<dim3((unsigned)((max_total + 255) / 256), nl), 256, 0, s>>>(a);
    csc_scan_kernel<<<dim3(p.bh, nl), kScanThreads, 0, s>>>(a);
    csc_fill_kernel<<<dim3((unsigned)((max_total + 255) / 256), nl), 256, 0, s>>>(a);
    csc_sort_kernel<<<dim3((unsigned)((max_total + 255) / 256), nl), 256, 0, s>>>(a);
    if (p.n[1] > kLongList)                                 // level 0 has the most rows; no list is longer than its level's rows
        csc_sort_long_kernel<<<dim3((unsigned)((max_nk + 255) / 256), nl), 256, 0, s>>>(a);
    return hipGetLastError();
}

// --------------------------------------------------------------------------------------- dQ (scalar path)
// Query-major: same list walk as the forward; P recomputed from the saved logsumexp.
template <class T>
__global__ void __launch_bounds__(256) dq_generic(LevelTable t, const T *Q, const T *dO, const float *LSE,
                                                   const float *D, T *dQ, int64_t N, int64_t total_rows) {
    __shared__ float qs[4][128], gs[4][128];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, d = t.d;
    int64_t row = (int64_t)blockIdx.x * 4 + wave;
    const bool active = row < total_rows;
    if (!active) row = total_rows - 1;
    const int64_t bh = row / N, q = row % N, blk = q / t.B;
    for (int c = lane; c < d; c += 64) { qs[wave][c] = to_f(Q[row * d + c]); gs[wave][c] = to_f(dO[row * d + c]); }
    __syncthreads();
    const float lse = LSE[row], delta = D[row];
    const int M = t.seg[t.nlev];
    float acc0 = 0.f, acc1 = 0.f;
    for (int base = 0; base < M; base += 64) {
        const int pos = base + lane;
        int lev = 0, tok = 0;
        float ds = 0.f;
        if (pos < M) {
            list_entry(t, bh, blk, pos, lev, tok);
            const int64_t off = (bh * t.n[lev] + tok) * d;
            const float z = t.scale * dot_row<T>(static_cast<const T *>(t.K[lev]) + off, qs[wave], d) + t.bias[lev];
            const float pr = expf(z - lse);
            const float dp = dot_row<T>(static_cast<const T *>(t.V[lev]) + off, gs[wave], d);
            ds = pr * (dp - delta);
        }
        const int cnt = min(64, M - base);
        for (int j = 0; j < cnt; ++j) {
            const float dj = __shfl(ds, j, 64);
            const int lj = __shfl(lev, j, 64), tj = __shfl(tok, j, 64);
            const T *k = static_cast<const T *>(t.K[lj]) + (bh * t.n[lj] + tj) * d;
            if (lane < d) acc0 = fmaf(dj, to_f(k[lane]), acc0);
            if (lane + 64 < d) acc1 = fmaf(dj, to_f(k[lane + 64]), acc1);
        }
    }
    if (active) {
        if (lane < d) dQ[row * d + lane] = from_f<T>(t.scale * acc0);
        if (lane + 64 < d) dQ[row * d + lane + 64] = from_f<T>(t.scale * acc1);
    }
}

hipError_t launch_dq_generic(const Plan &p, const LevelTable &t, const void *Q, const void *dO, const float *LSE,
                             const float *D, void *dQ, hipStream_t s) {
    const int64_t rows = (int64_t)p.bh * p.N;
    dim3 grid((unsigned)((rows + 3) / 4));
    if (p.elt == 4)
        dq_generic<float><<<grid, 256, 0, s>>>(t, (const float *)Q, (const float *)dO, LSE, D, (float *)dQ, p.N, rows);
    else
        dq_generic<bf16_t><<<grid, 256, 0, s>>>(t, (const bf16_t *)Q, (const bf16_t *)dO, LSE, D, (bf16_t *)dQ, p.N,
                                                rows);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------ dK, dV (scalar path)
// Key-major (Sec. 4.3): one wave per level-l key token walks the query blocks that listed its block
// (lists from Alg. 2; at the coarsest enriched level L every query).  Level >= 1 results go to fp32
// buffers; level 0 adds its parent's share (adjoint of mean pooling) and rounds once to the I/O type.
template <class T>
__global__ void __launch_bounds__(256) dkv_generic(LevelTable t, int l, const T *Q, const T *dO, const float *LSE,
                                                    const float *D, const int32_t *C, const int32_t *Iq,
                                                    float *dKacc, float *dVacc, const float *parK, const float *parV,
                                                    T *dK, T *dV, int64_t N, int64_t total_tokens) {
    __shared__ float ks[4][128], vs[4][128];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, d = t.d, B = t.B;
    int64_t tf = (int64_t)blockIdx.x * 4 + wave;           // flat key token over bh * n_l
    const bool active = tf < total_tokens;
    if (!active) tf = total_tokens - 1;
    const int64_t n_l = t.n[l], bh = tf / n_l, tok = tf % n_l;
    const T *Kl = static_cast<const T *>(t.K[l]), *Vl = static_cast<const T *>(t.V[l]);
    for (int c = lane; c < d; c += 64) { ks[wave][c] = to_f(Kl[tf * d + c]); vs[wave][c] = to_f(Vl[tf * d + c]); }
    __syncthreads();
    const bool dense = (l == t.L);
    const int64_t span = dense ? 1 : t.Bpow[l + 1];        // fine queries per listed query block
    int64_t qcount;
    const int32_t *lst = nullptr;
    if (dense) {
        qcount = N;
    } else {
        const int64_t T_keys = t.rows[l], j = tok / B;
        const int32_t beg = C[bh * (T_keys + 1) + j], end = C[bh * (T_keys + 1) + j + 1];
        lst = Iq + bh * T_keys * t.Kl[l] + beg;
        qcount = (int64_t)(end - beg) * span;
    }
    float dk0 = 0.f, dk1 = 0.f, dv0 = 0.f, dv1 = 0.f;
    for (int64_t base = 0; base < qcount; base += 64) {
        const int64_t g = base + lane;
        float pr = 0.f, ds = 0.f;
        int64_t qrow = 0;
        if (g < qcount) {
            const int64_t q = dense ? g : (int64_t)lst[g / span] * span + g % span;
            qrow = bh * N + q;
            const float z = t.scale * dot_row<T>(Q + qrow * d, ks[wave], d) + t.bias[l];
            pr = expf(z - LSE[qrow]);
            const float dp = dot_row<T>(dO + qrow * d, vs[wave], d);
            ds = pr * (dp - D[qrow]);
        }
        const int cnt = (int)min((int64_t)64, qcount - base);
        for (int j = 0; j < cnt; ++j) {
            const float pj = __shfl(pr, j, 64), dj = __shfl(ds, j, 64);
            const int64_t rj = __shfl(qrow, j, 64);
            if (lane < d) {
                dv0 = fmaf(pj, to_f(dO[rj * d + lane]), dv0);
                dk0 = fmaf(dj, to_f(Q[rj * d + lane]), dk0);
            }
            if (lane + 64 < d) {
                dv1 = fmaf(pj, to_f(dO[rj * d + lane + 64]), dv1);
                dk1 = fmaf(dj, to_f(Q[rj * d + lane + 64]), dk1);
            }
        }
    }
    if (!active) return;
    dk0 *= t.scale; dk1 *= t.scale;
    if (l > 0) {
        if (lane < d) { dKacc[tf * d + lane] = dk0; dVacc[tf * d + lane] = dv0; }
        if (lane + 64 < d) { dKacc[tf * d + lane + 64] = dk1; dVacc[tf * d + lane + 64] = dv1; }
    } else {
        const float invB = 1.f / (float)B;
        const int64_t par = (bh * t.n[1] + tok / B) * d;   // parent token at level 1
        if (lane < d) {
            const float pk = parK ? parK[par + lane] * invB : 0.f, pv = parV ? parV[par + lane] * invB : 0.f;
            dK[tf * d + lane] = from_f<T>(dk0 + pk);
            dV[tf * d + lane] = from_f<T>(dv0 + pv);
        }
        if (lane + 64 < d) {
            const float pk = parK ? parK[par + lane + 64] * invB : 0.f, pv = parV ? parV[par + lane + 64] * invB : 0.f;
            dK[tf * d + lane + 64] = from_f<T>(dk1 + pk);
            dV[tf * d + lane + 64] = from_f<T>(dv1 + pv);
        }
    }
}

hipError_t launch_dkv_generic(const Plan &p, const LevelTable &t, int l, const void *Q, const void *dO,
                              const float *LSE, const float *D, void *ws, void *dK, void *dV, hipStream_t s) {
    char *w = static_cast<char *>(ws);
    const int64_t total = (int64_t)p.bh * p.n[l];
    dim3 grid((unsigned)((total + 3) / 4));
    const int32_t *C = l < p.L ? (const int32_t *)(w + p.C_off[l]) : nullptr;
    const int32_t *Iq = l < p.L ? (const int32_t *)(w + p.Iq_off[l]) : nullptr;
    float *ka = l > 0 ? (float *)(w + p.dKacc_off[l]) : nullptr, *va = l > 0 ? (float *)(w + p.dVacc_off[l]) : nullptr;
    const bool has_parent = (l == 0 && p.Le >= 1);
    const float *pk = has_parent ? (const float *)(w + p.dKacc_off[1]) : nullptr;
    const float *pv = has_parent ? (const float *)(w + p.dVacc_off[1]) : nullptr;
    if (p.elt == 4)
        dkv_generic<float><<<grid, 256, 0, s>>>(t, l, (const float *)Q, (const float *)dO, LSE, D, C, Iq, ka, va, pk, pv,
                                                (float *)dK, (float *)dV, p.N, total);
    else
        dkv_generic<bf16_t><<<grid, 256, 0, s>>>(t, l, (const bf16_t *)Q, (const bf16_t *)dO, LSE, D, C, Iq, ka, va, pk,
                                                 pv, (bf16_t *)dK, (bf16_t *)dV, p.N, total);
    return hipGetLastError();
}

// ------------------------------------------------------- key-major lists through a dense block mask (comparator)
// The mask-based baseline of Sec. 5.4 ("Efficient Backward Implementation", Fig. 4): the row-major lists I^(0) are
// turned into a dense binary T x T block mask and the key/value backward scans it, skipping the unmarked blocks.
// Here the mask is kept key-major (mask[key block][query block], one byte each: the layout that makes the scan a
// contiguous read, the baseline's best case), and the scan of a key block's row writes the marked query blocks, in
// ascending order, as that key's list -- the same (C, Iq) pair Alg. 2 produces in O(T K) -- so that the very same
// dK / dV kernel runs behind both.  Work and memory of this path are O(T^2) per head.
__global__ void __launch_bounds__(256) mask_zero_kernel(uint4 *mask16, int64_t n16) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) mask16[i] = make_uint4(0u, 0u, 0u, 0u);
}
// one thread per entry of I^(0): marks (key, query block) and counts the key's listers
__global__ void __launch_bounds__(256) mask_mark_kernel(const int32_t *I, uint8_t *mask, int32_t *cnt, int64_t T, int Kl,
                                                        int64_t total) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int64_t eph = T * Kl, bh = e / eph, row = (e % eph) / Kl;
    const int32_t key = I[e];
    mask[(bh * T + key) * T + row] = 1;
    atomicAdd(&cnt[bh * T + key], 1);
}
// one wave per key block: scans its T mask bytes, 1024 at a time, and appends the marked query blocks to its list
__global__ void __launch_bounds__(256) mask_scan_kernel(const uint8_t *mask, const int32_t *C, int32_t *Iq, int64_t T,
                                                        int64_t eph, int64_t nk) {
    const int lane = threadIdx.x & 63;
    const int64_t kb = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);           // flat key block over (batch, head)
    if (kb >= nk) return;
    const int64_t bh = kb / T, key = kb % T;
    const uint8_t *row = mask + kb * T;
    int32_t *dst = Iq + bh * eph + C[bh * (T + 1) + key];
    int written = 0;
    for (int64_t base = 0; base < T; base += 1024) {
        const int64_t i0 = base + 16 * lane;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (i0 + 16 <= T) v = *reinterpret_cast<const uint4 *>(row + i0);
        else for (int k = 0; k < 16 && i0 + k < T; ++k) reinterpret_cast<uint8_t *>(&v)[k] = row[i0 + k];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        int mine = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) mine += __popc(w[k] & 0x01010101u);
        int incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o, 64);
            if (lane >= o) incl += y;
        }
        int pos = written + incl - mine;
#pragma unroll
        for (int k = 0; k < 16; ++k)
            if ((w[k >> 2] >> (8 * (k & 3))) & 1u) dst[pos++] = (int32_t)(i0 + k);
        written += __shfl(incl, 63, 64);
    }
}

// Level 0's key-major lists through the dense mask: C and Iq of level 0 in the backward workspace, as launch_csc.
hipError_t launch_mask_lists(const Plan &p, const int32_t *indices, void *ws, void *mask, hipStream_t s) {
    char *w = static_cast<char *>(ws);
    const int64_t T = p.n[1], nk = T * p.bh, eph = T * p.Kl[0], total = eph * p.bh;
    CscLevels a;
    CscLevel &L = a.lv[0];
    L.T = T; L.Kl = p.Kl[0]; L.eph = eph; L.total = total; L.nk = nk;
    L.I = reinterpret_cast<const int32_t *>(reinterpret_cast<const char *>(indices) + p.idx_off[0]);
    L.cnt = (int32_t *)(w + p.cnt_off[0]);
    L.C = (int32_t *)(w + p.C_off[0]);
    L.Iq = (int32_t *)(w + p.Iq_off[0]);
    L.Iq_tmp = (int32_t *)(w + p.Iqtmp_off[0]);
    const int64_t n16 = (nk * T + 15) / 16;
    if (n16 / 256 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    mask_zero_kernel<<<dim3((unsigned)((n16 + 255) / 256)), 256, 0, s>>>(static_cast<uint4 *>(mask), n16);
    csc_zero_kernel<<<dim3((unsigned)((nk + 255) / 256), 1), 256, 0, s>>>(a);
    mask_mark_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, s>>>(L.I, static_cast<uint8_t *>(mask), L.cnt, T, L.Kl, total);
    csc_scan_kernel<<<dim3(p.bh, 1), kScanThreads, 0, s>>>(a);
    mask_scan_kernel<<<dim3((unsigned)((nk + 3) / 4)), 256, 0, s>>>(static_cast<const uint8_t *>(mask), L.C, L.Iq, T, eph, nk);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ un-pool
// Adjoint of one pooling step on the fp32 gradient buffers: level l-1 token t*B + r gains (1/B) of level-l
// token t (l >= 2 here; the step into level 0 is folded into the level-0 dK/dV epilogue).
__global__ void __launch_bounds__(256) unpool_kernel(float *dstK, float *dstV, const float *srcK, const float *srcV,
                                                     int64_t total, int d, int B) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int64_t tok = i / d, c = i % d;
    const int64_t src = (tok / B) * d + c;                 // flat over bh: n_{l-1} = B * n_l per head
    const float invB = 1.f / (float)B;
    dstK[i] += srcK[src] * invB;
    dstV[i] += srcV[src] * invB;
}

hipError_t launch_unpool(const Plan &p, int l, void *ws, hipStream_t s) {
    char *w = static_cast<char *>(ws);
    const int64_t total = (int64_t)p.bh * p.n[l - 1] * p.d;
    unpool_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(
        (float *)(w + p.dKacc_off[l - 1]), (float *)(w + p.dVacc_off[l - 1]), (const float *)(w + p.dKacc_off[l]),
        (const float *)(w + p.dVacc_off[l]), total, p.d, p.B);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------- index reordering (Sec. 5.1)
// Tokens of a W x W pixel grid in nested-patch order: token t is the pixel whose x / y are the even / odd bits
// of t, so every aligned run of 4^i tokens is one aligned 2^i x 2^i patch.  One thread per 16-byte chunk of a
// row; forward: out[t] = in[y W + x], inverse: out[y W + x] = in[t].
__global__ void __launch_bounds__(256) reorder_kernel(const uint4 *in, uint4 *out, int64_t N, int cpr, int bits,
                                                       int inverse, int64_t total) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int64_t row = idx / cpr, bh = row / N, t = row % N;
    const int c = (int)(idx % cpr);
    int64_t x = 0, y = 0;
    for (int b = 0; b < bits; ++b) {
        x |= ((t >> (2 * b)) & 1) << b;
        y |= ((t >> (2 * b + 1)) & 1) << b;
    }
    const int64_t r = (y << bits) + x;
    const int64_t src = inverse ? t : r, dst = inverse ? r : t;
    out[(bh * N + dst) * cpr + c] = in[(bh * N + src) * cpr + c];
}

hipError_t launch_reorder(int64_t bh, int64_t N, int row_bytes, int bits, int inverse, const void *in, void *out,
                          hipStream_t s) {
    const int cpr = row_bytes / 16;
    const int64_t total = bh * N * cpr;
    reorder_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint4 *)in, (uint4 *)out, N, cpr, bits, inverse,
                                                                   total);
    return hipGetLastError();
}

}  // namespace llsa
