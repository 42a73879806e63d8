// Device helpers shared by the bf16 MFMA kernels (gfx950): vector types, the 16x16x32 bf16 MFMA, the LDS
// transpose read and the walk over the 16-token key blocks of a query block's gathered list.
//
// Register layouts of v_mfma_f32_16x16x32_bf16 (lane = 16*g + i, g = 0..3, i = 0..15):
//   A (16 x 32): lane holds row i,    contraction slots 8g .. 8g+7
//   B (32 x 16): lane holds column i, contraction slots 8g .. 8g+7
//   D (16 x 16): lane holds column i, rows 4g .. 4g+3
// ds_read_b64_tr_b16 (per block of 16 lanes, lane r supplies the address of 4 consecutive 16-bit
// values): output lane i, element e = element (i % 4) of the chunk addressed by lane 4e + i / 4.
#pragma once
#include "llsa_internal.h"

namespace llsa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#define LLSA_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 ld_bf16x8(const void *p) { return *reinterpret_cast<const bf16x8 *>(p); }

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t bf16_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) { return bf16_bits(lo) | (bf16_bits(hi) << 16); }

__device__ __forceinline__ bf16x8 pack8(const f32x4 &a, const f32x4 &b) {
    union { uint32_t u[4]; bf16x8 v; } r;
    r.u[0] = pack_bf16(a[0], a[1]); r.u[1] = pack_bf16(a[2], a[3]);
    r.u[2] = pack_bf16(b[0], b[1]); r.u[3] = pack_bf16(b[2], b[3]);
    return r.v;
}

// Two transposing LDS reads glued into one 8-slot MFMA operand.
__device__ __forceinline__ bf16x8 lds_tr_pair(const char *lo, const char *hi) {
    union { s16x4 h[2]; bf16x8 v; } r;
    r.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LLSA_LDS s16x4 *)(lo));
    r.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LLSA_LDS s16x4 *)(hi));
    return r.v;
}

// arr[idx] for a small kernel-argument array without dynamic indexing (which would spill the table to
// scratch memory): a chain of selects over compile-time positions.
template <class T, int n>
__device__ __forceinline__ T pick(const T (&arr)[n], int idx) {
    T v = arr[0];
#pragma unroll
    for (int j = 1; j < n; ++j) v = (idx == j) ? arr[j] : v;
    return v;
}

// One 16-token key block of a gathered list.
struct KeyBlock {
    const uint16_t *K, *V;   // first row of the block in its level's key / value tensor
    float bias2;             // log2 of the level's token weight
    int cnt;                 // valid tokens (16, or fewer in the last block of the coarsest level; 0 = no block)
};

// Walks the key blocks of fine query block `blk` of head `bh` in list order (Alg. 1, enrichment loop),
// for B = 16.  Everything here is wave-uniform.
struct BlockWalker {
    const LevelTable &t;
    int64_t bh, blk;
    int l, k, nk;
    __device__ BlockWalker(const LevelTable &tab, int64_t bh_, int64_t blk_) : t(tab), bh(bh_), blk(blk_), l(0), k(0) {
        nk = count(0);
    }
    __device__ int count(int lev) const {
        if (lev >= t.nlev) return 0;
        return lev < t.L ? pick(t.Kl, lev) : (int)((pick(t.n, lev) + 15) >> 4);
    }
    __device__ bool done() const { return l >= t.nlev; }
    // d = head dimension; an exhausted walker returns cnt = 0 and null pointers
    __device__ KeyBlock next(int d) {
        KeyBlock b;
        if (done()) { b.K = b.V = nullptr; b.bias2 = 0.f; b.cnt = 0; return b; }
        const int64_t n_l = pick(t.n, l);
        int64_t tok0;
        if (l < t.L) {
            const int64_t row = blk / pick(t.Bpow, l);
            const int kl = pick(t.Kl, l);
            tok0 = (int64_t)pick(t.I, l)[(bh * pick(t.rows, l) + row) * kl + k] * 16;
            b.cnt = 16;
        } else {
            tok0 = k * 16;
            b.cnt = min(16, (int)n_l - k * 16);
        }
        const int64_t off = (bh * n_l + tok0) * d;
        b.K = static_cast<const uint16_t *>(pick(t.K, l)) + off;
        b.V = static_cast<const uint16_t *>(pick(t.V, l)) + off;
        b.bias2 = pick(t.bias, l) * 1.4426950408889634f;
        if (++k == nk) { ++l; k = 0; nk = count(l); }
        return b;
    }
};

}  // namespace llsa
