// Device helpers shared by the bf16 MFMA kernels (gfx950): vector types, the 16x16x32 bf16 MFMA, the LDS
// transpose read, cross-row reductions and the table of 16-token key blocks of a query block's list.
//
// Register layouts of v_mfma_f32_16x16x32_bf16 (lane = 16*g + i, g = 0..3, i = 0..15):
//   A (16 x 32): lane holds row i,    contraction slots 8g .. 8g+7
//   B (32 x 16): lane holds column i, contraction slots 8g .. 8g+7
//   D (16 x 16): lane holds column i, rows 4g .. 4g+3
// ds_read_b64_tr_b16 (per block of 16 lanes, lane r supplies the address of 4 consecutive 16-bit
// values): output lane i, element e = element (i % 4) of the chunk addressed by lane 4e + i / 4.
// v_permlane16_swap / v_permlane32_swap with both operands equal to x return {x[l], x[l ^ 16]} resp.
// {x[l], x[l ^ 32]} (in some order) in every lane l.
#pragma once
#include "llsa_internal.h"

namespace llsa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

#define LLSA_LDS __attribute__((address_space(3)))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 ld_bf16x8(const void *p) { return *reinterpret_cast<const bf16x8 *>(p); }

// two fp32 -> packed bf16 (round to nearest even; one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    union { bf16x2 v; uint32_t u; } r;
    r.v[0] = (__bf16)lo;
    r.v[1] = (__bf16)hi;
    return r.u;
}

__device__ __forceinline__ bf16x8 pack8(const f32x4 &a, const f32x4 &b) {
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) { r[i] = (__bf16)a[i]; r[4 + i] = (__bf16)b[i]; }
    return r;
}

// Two transposing LDS reads glued into one 8-slot MFMA operand.
__device__ __forceinline__ bf16x8 lds_tr_pair(const char *lo, const char *hi) {
    union { s16x4 h[2]; bf16x8 v; } r;
    r.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LLSA_LDS s16x4 *)(lo));
    r.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LLSA_LDS s16x4 *)(hi));
    return r.v;
}

// All-reduce over the four lanes {i, i+16, i+32, i+48} (the four row groups of one MFMA column).
__device__ __forceinline__ float rows_max(float x) {
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows_sum(float x) {
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(y), __float_as_uint(y), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
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

// Rows of D bf16 kept unpadded in LDS, the 16-byte chunk c of row r stored at chunk c ^ swz_key(r).
// d = 64 (128-byte rows, half a row of the 64 LDS banks): the key gives 16 consecutive rows 8 distinct values per
// row parity, so the row-wise 16-byte reads of 16 lanes hit 16 different bank groups.  (A key that also spreads the
// transposed 8-byte reads of a half wave was timed: those reads did not get faster, the row-wise ones got slower.)
// d = 128 (256-byte rows, all banks): the key is a bijection of 16 consecutive rows onto the 16 chunks, and its
// upper three bits differ among the 8 rows a half wave reads transposed.
template <int D> __device__ __forceinline__ int swz_key(int r) {
    return D == 64 ? ((r >> 1) & 7) : (((r & 7) << 1) | ((r >> 3) & 1));
}

// Per-lane byte offsets of the MFMA operand reads inside a 16-row slice of such unpadded, swizzled rows (2 D bytes
// each): row[ks] = the 16-byte row-wise read of row lane % 16, contraction step ks (A or B operand with the rows as
// the 16-wide dimension); tr[n] = the address a lane supplies to the transposing 64-bit read for the n-th group of 16
// channels (rows 4 (lane / 16) + (lane % 16) / 4).  The swizzle key of a row depends on the lane only.
template <int D> struct TileOffsets { int row[D / 32], tr[D / 16]; };
template <int D> __device__ __forceinline__ TileOffsets<D> tile_offsets(int lane) {
    constexpr int ROWB = 2 * D;
    const int i16 = lane & 15, g = lane >> 4;
    const int key_row = swz_key<D>(i16), key_tr = swz_key<D>(4 * g + (i16 >> 2));
    TileOffsets<D> o;
#pragma unroll
    for (int ks = 0; ks < D / 32; ++ks) o.row[ks] = i16 * ROWB + (((g + 4 * ks) ^ key_row) << 4);
#pragma unroll
    for (int n = 0; n < D / 16; ++n)
        o.tr[n] = (4 * g + (i16 >> 2)) * ROWB + (((2 * n + ((i16 >> 1) & 1)) ^ key_tr) << 4) + ((i16 & 1) << 3);
    return o;
}

// Workgroup id -> work item so that the workgroups one XCD receives (ids congruent modulo 8) cover a
// contiguous range of work items: neighbouring query blocks gather overlapping keys, which then stay in
// that XCD's L2.
__device__ __forceinline__ int64_t xcd_contiguous(int64_t w, int64_t total) {
    const int64_t per = total >> 3;
    return (w < per * 8) ? (w & 7) * per + (w >> 3) : w;
}

// The 16-token key tiles of one 16-query tile's list (Alg. 1, enrichment loop), 64 at a time: lane j of the wave
// describes tile 64 * chunk + j.  A listed block of B = 16 * 2^ls tokens is 2^ls consecutive tiles; query tile `blk`
// (queries 16 blk ...) reads row 16 blk / B^(l+1) of I^(l).  The main loops fetch a block's fields with
// v_readlane (block numbers are wave-uniform), which keeps the per-tile scalar work small.
struct BlockTable {
    uint64_t kptr, vptr;     // address of the block's first key / value row
    float bias2;             // log2 of the level's token weight
    int cnt;                 // valid rows: 16, fewer in the last block of a ragged coarsest level, 0 past the end

    // lane j describes list block base + 64 * chunk + j; only levels below lev_end are looked at
    __device__ __forceinline__ void fill(const LevelTable &t, int64_t bh, int64_t blk, int base, int chunk, int lane,
                                         int d, int lev_end = kMaxL + 1) {
        const int jb = base + chunk * 64 + lane;
        kptr = vptr = 0;
        bias2 = 0.f;
        cnt = 0;
        const int nl = min(t.nlev, lev_end);
        for (int l = 0; l < nl; ++l) {                           // wave-uniform loop over the levels in the list
            const int b0 = pick(t.bseg, l), b1 = pick(t.bseg, l + 1);
            const int64_t n_l = pick(t.n, l);
            const char *Kb = static_cast<const char *>(pick(t.K, l)), *Vb = static_cast<const char *>(pick(t.V, l));
            if (jb >= b0 && jb < b1) {
                const int k = jb - b0;
                int64_t tok0;
                if (l < t.L) {
                    const int64_t row = blk >> (t.lb * (l + 1) - 4);
                    const int32_t listed = pick(t.I, l)[(bh * pick(t.rows, l) + row) * pick(t.Kl, l) + (k >> t.ls)];
                    tok0 = ((int64_t)listed << t.lb) + ((k & ((1 << t.ls) - 1)) << 4);
                    cnt = 16;
                } else {
                    tok0 = (int64_t)k * 16;
                    cnt = min(16, (int)(n_l - tok0));
                }
                const int64_t off = (bh * n_l + tok0) * d * 2;
                kptr = reinterpret_cast<uint64_t>(Kb + off);
                vptr = reinterpret_cast<uint64_t>(Vb + off);
                bias2 = pick(t.bias, l) * kLog2e;
            }
        }
    }
    // The same table for every wave of a workgroup (same head, same list rows): wave 0 builds it, the others copy it
    // from `tab` (64 x 24 bytes of LDS nobody else uses meanwhile).  Every thread of the workgroup must call this.
    __device__ __forceinline__ void fill_once(const LevelTable &t, int64_t bh, int64_t blk, int base, int lane, int wave,
                                              int d, uint32_t *tab) {
        if (wave == 0) {
            fill(t, bh, blk, base, 0, lane, d);
            tab[lane] = (uint32_t)kptr;
            tab[64 + lane] = (uint32_t)(kptr >> 32);
            tab[128 + lane] = (uint32_t)vptr;
            tab[192 + lane] = (uint32_t)(vptr >> 32);
            tab[256 + lane] = __float_as_uint(bias2);
            tab[320 + lane] = (uint32_t)cnt;
        }
        __syncthreads();
        if (wave != 0) {
            kptr = ((uint64_t)tab[64 + lane] << 32) | tab[lane];
            vptr = ((uint64_t)tab[192 + lane] << 32) | tab[128 + lane];
            bias2 = __uint_as_float(tab[256 + lane]);
            cnt = (int)tab[320 + lane];
        }
    }
    static __device__ __forceinline__ const char *rl_ptr(uint64_t v, int j) {
        const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, j);
        const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), j);
        return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
    }
    __device__ __forceinline__ const char *K(int j) const { return rl_ptr(kptr, j); }
    __device__ __forceinline__ const char *V(int j) const { return rl_ptr(vptr, j); }
    __device__ __forceinline__ int count(int j) const { return __builtin_amdgcn_readlane(cnt, j); }
    __device__ __forceinline__ float bias(int j) const {
        return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(bias2), j));
    }
};

}  // namespace llsa
