// Device code shared by the LoRA kernels of libtidal (included by the .hip files only).
#ifndef TIDAL_LORA_DEVICE_H_
#define TIDAL_LORA_DEVICE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "tidal_internal.h"

namespace tidal {

// Pointers that reach a kernel through a descriptor in memory are generic to the compiler, and
// generic accesses become flat_load/flat_store, which also occupy the LDS path and its counter.
// Everything these kernels touch outside LDS is global memory, so say so.
#define TIDAL_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ TIDAL_GLOBAL T* as_global(T* p) {
    return (TIDAL_GLOBAL T*)p;
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef float f32x2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------
// Packed factor layouts ("operand order")
// ---------------------------------------------------------------------------------------
// The device copy of an adapter keeps A and B as 16-byte groups of 8 consecutive ranks, ordered so
// that the matrix-core operand a wave needs is one contiguous kilobyte, lane after lane:
//   At (A transposed, in rounded up to 256 columns, ranks padded to rp = 16*KS with zeros):
//       group of column j, ranks 16*ks + 8*kg .. +8  at index
//       (((j / 256) * 8 + j % 8) * KS + ks) * 64 + kg * 32 + (j % 256) / 8
//     i.e. per strip of 256 columns, per T = j % 8, per ks: the 64 lanes (n = (j % 256) / 8, kg) of
//     the MFMA B operand of tile T;
//   Bp (out rounded up to 32 rows): group of row i, same ranks, at
//       ((i / 32) * KS + ks) * 64 + kg * 32 + i % 32
//     i.e. per block of 32 rows, per ks: the 64 lanes (m = i % 32, kg) of the MFMA A operand.
// With plain row-major factors every lane of such a load touched a cache line of its own (64 cache
// accesses per instruction against 16 for a load of W), and at 64 ranks the factor loads were 60 %
// of all accesses of the texture-address path, which was busy 88 % of the time: the in-place pass
// was bound there, not by HBM.  Padding entries hold zeros, so loads need no clamping.
__host__ __device__ __forceinline__ int64_t at_group(int64_t j, int ks, int kg, int KS) {
    return (((j >> 8) * 8 + (j & 7)) * KS + ks) * 64 + kg * 32 + ((j & 255) >> 3);
}
__host__ __device__ __forceinline__ int64_t bp_group(int64_t i, int ks, int kg, int KS) {
    return ((i >> 5) * KS + ks) * 64 + kg * 32 + (i & 31);
}

// Two adjacent bf16 of W (one 32-bit word, low half = lower column) += s * (d_lo, d_hi).
// The narrowing is v_cvt_pk_bf16_f32: round to nearest even, subnormals kept, NaN quieted with
// sign and upper payload kept -- bit-identical to the integer formula
// (u + 0x7FFF + ((u >> 16) & 1)) >> 16 for every one of the 2^32 inputs (checked on gfx950).
__device__ __forceinline__ uint32_t rmw2(uint32_t w2, float d_lo, float d_hi, float s) {
    const float w_lo = __uint_as_float(w2 << 16);
    const float w_hi = __uint_as_float(w2 & 0xFFFF0000u);
    const f32x2 r = {__builtin_fmaf(s, d_lo, w_lo), __builtin_fmaf(s, d_hi, w_hi)};
    const bf16x2 b = __builtin_convertvector(r, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// ---------------------------------------------------------------------------------------
// Matrix-core kernel
// ---------------------------------------------------------------------------------------

template <int NT> struct RowVec;     // the NT adjacent bf16 a lane owns in one row
template <> struct RowVec<2> { typedef uint32_t type; };
template <> struct RowVec<4> { typedef u32x2 type; };
template <> struct RowVec<8> { typedef u32x4 type; };

template <int NT>
__device__ __forceinline__ void unpack_words(const typename RowVec<NT>::type& v, uint32_t (&w)[NT / 2]) {
    if constexpr (NT == 2) { w[0] = v; }
    else if constexpr (NT == 4) { w[0] = v.x; w[1] = v.y; }
    else { w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w; }
}

template <int NT>
__device__ __forceinline__ typename RowVec<NT>::type pack_words(const uint32_t (&w)[NT / 2]) {
    typename RowVec<NT>::type v;
    if constexpr (NT == 2) { v = w[0]; }
    else if constexpr (NT == 4) { v.x = w[0]; v.y = w[1]; }
    else { v.x = w[0]; v.y = w[1]; v.z = w[2]; v.w = w[3]; }
    return v;
}

// Columns of A for the lane's NT columns: MFMA B operand, K x N with N index n = lane % 32 and
// k = 16*ks + 8*(lane / 32) + 0..7; the lane's column of tile T is j0 + NT*n + T.  With NT = 8 and
// j0 a multiple of 256 every load is one contiguous kilobyte.
template <int NT, int KS>
__device__ __forceinline__ void load_strip(const uint16_t* __restrict__ At, int j0, int lane,
                                           bf16x8 (&bop)[NT][KS ? KS : 1]) {
    if constexpr (KS > 0) {
        const int n = lane & 31, kg = lane >> 5;
        const TIDAL_GLOBAL bf16x8* g = as_global((const bf16x8*)At);
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            const int64_t base = at_group(j0 + NT * n + T, 0, kg, KS);     // columns past `in` are zero padding
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) bop[T][ks] = g[base + 64 * ks];
        }
    }
}

// The same operand from a row-major matrix of `lines` rows x 16*KS bf16 (row j = one column of the
// operand): the expand step of the unmerged apply, whose strip is rows of B.
template <int NT, int KS>
__device__ __forceinline__ void load_strip_rows(const uint16_t* __restrict__ M, int lines, int j0, int lane,
                                                bf16x8 (&bop)[NT][KS ? KS : 1]) {
    if constexpr (KS > 0) {
        const int n = lane & 31, kg = lane >> 5;
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            int j = j0 + NT * n + T;
            j = j < lines ? j : lines - 1;                 // ragged strip: clamp, masked at the store
            const uint16_t* p = M + (int64_t)j * (16 * KS) + 8 * kg;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) bop[T][ks] = *as_global((const bf16x8*)(p + 16 * ks));
        }
    }
}

// Rows i0 .. i0+31 of B as the MFMA A operand (lane: row lane % 32, ranks 8*(lane / 32) + 0..7 of
// each 16): one contiguous kilobyte per 16 ranks when i0 is a multiple of 32.
template <int KS>
__device__ __forceinline__ void load_b_rows(const uint16_t* __restrict__ Bp, int i0, int lane, bf16x8 (&aop)[KS ? KS : 1]) {
    if constexpr (KS > 0) {
        const TIDAL_GLOBAL bf16x8* g = as_global((const bf16x8*)Bp);
        const int64_t base = bp_group(i0 + (lane & 31), 0, lane >> 5, KS);   // rows past `out` are zero padding
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) aop[ks] = g[base + 64 * ks];
    }
}

// The same operand from a row-major matrix of `rows` rows x 16*KS bf16 (the rank-space intermediate
// of the unmerged apply).
template <int KS>
__device__ __forceinline__ void load_rows(const uint16_t* __restrict__ M, int rows, int i0, int lane,
                                          bf16x8 (&aop)[KS ? KS : 1]) {
    if constexpr (KS > 0) {
        int m = i0 + (lane & 31);
        m = m < rows ? m : rows - 1;
        const uint16_t* p = M + (int64_t)m * (16 * KS) + 8 * (lane >> 5);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) aop[ks] = *as_global((const bf16x8*)(p + 16 * ks));
    }
}

// delta tile for one adapter: acc[T][v] = sum_k B[i0 + row(v)][k] * A[k][j0 + NT*n + T]
template <int NT, int KS>
__device__ __forceinline__ void delta_tile(const bf16x8 (&aop)[KS ? KS : 1], const bf16x8 (&bop)[NT][KS ? KS : 1],
                                           f32x16 (&acc)[NT]) {
    if constexpr (KS > 0) {
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            f32x16 c = {0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], bop[T][ks], c, 0, 0, 0);
            acc[T] = c;
        }
    }
}

template <int NT>
__device__ __forceinline__ void apply_tile(uint32_t (&w)[16][NT / 2], const f32x16 (&acc)[NT], float s) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
#pragma unroll
        for (int p = 0; p < NT / 2; ++p) w[v][p] = rmw2(w[v][p], acc[2 * p][v], acc[2 * p + 1][v], s);
}

// delta_tile and apply_tile in one: the tiles are produced two at a time (the two adjacent columns
// of one 32-bit word of W) and consumed at once, so only 32 accumulator registers are live instead
// of 16 * NT.  That is what lets two waves share a SIMD for the small ranks.
template <int NT, int KS>
__device__ __forceinline__ void delta_apply(const uint16_t* __restrict__ Bp, int i0, int lane,
                                            const bf16x8 (&bop)[NT][KS ? KS : 1], uint32_t (&w)[16][NT / 2], float s) {
    if constexpr (KS > 0) {
        bf16x8 aop[KS];
        load_b_rows<KS>(Bp, i0, lane, aop);
#pragma unroll
        for (int q = 0; q < NT / 2; ++q) {
            f32x16 c0 = {0}, c1 = {0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], bop[2 * q][ks], c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], bop[2 * q + 1][ks], c1, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) w[v][q] = rmw2(w[v][q], c0[v], c1[v], s);
        }
    }
}

// W is touched exactly once per pass, so its accesses carry the non-temporal hint (measured:
// 4-6 % more bandwidth than plain accesses, the caches keep the A/B factors instead).
template <typename V>
__device__ __forceinline__ V load_w(const V* p) { return __builtin_nontemporal_load(as_global(p)); }
template <typename V>
__device__ __forceinline__ void store_w(V* p, V v) { __builtin_nontemporal_store(v, as_global(p)); }

// The lane's part of a 32-row block: 16 rows (8*(v/4) + 4*h + v%4), NT adjacent columns each.
// Interior blocks use one vector access per row; ragged ones go element by element.
template <int NT>
__device__ __forceinline__ void load_block(const uint16_t* __restrict__ W, int out, int in, int i0, int jl,
                                           int h, bool full, uint32_t (&w)[16][NT / 2]) {
    typedef typename RowVec<NT>::type vec_t;
    if (full) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
            vec_t x = load_w((const vec_t*)(W + (int64_t)row * in + jl));
            unpack_words<NT>(x, w[v]);
        }
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
#pragma unroll
            for (int p = 0; p < NT / 2; ++p) {
                uint32_t lo = 0, hi = 0;
                if (row < out && jl + 2 * p < in) lo = as_global(W)[(int64_t)row * in + jl + 2 * p];
                if (row < out && jl + 2 * p + 1 < in) hi = as_global(W)[(int64_t)row * in + jl + 2 * p + 1];
                w[v][p] = lo | (hi << 16);
            }
        }
    }
}

template <int NT>
__device__ __forceinline__ void store_block(uint16_t* __restrict__ W, int out, int in, int i0, int jl, int h,
                                            bool full, const uint32_t (&w)[16][NT / 2]) {
    typedef typename RowVec<NT>::type vec_t;
    if (full) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
            store_w((vec_t*)(W + (int64_t)row * in + jl), pack_words<NT>(w[v]));
        }
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
#pragma unroll
            for (int p = 0; p < NT / 2; ++p) {
                if (row < out && jl + 2 * p < in) as_global(W)[(int64_t)row * in + jl + 2 * p] = (uint16_t)(w[v][p] & 0xFFFFu);
                if (row < out && jl + 2 * p + 1 < in) as_global(W)[(int64_t)row * in + jl + 2 * p + 1] = (uint16_t)(w[v][p] >> 16);
            }
        }
    }
}

}  // namespace tidal
#endif
