// Materialisation with the adapter folded in.  gfx950 only.
//
// When a function's adapter is known while its weights stream in, the dynamic part of its
// initialisation (Sec. 5.2, adaptive template state reusing) needs no pass of its own: the kernel
// that turns a staged chunk into slot contents adds the adapter's delta before it rounds,
//     slot[i][j] = bf16( f32(src[i][j]) + s * sum_k B[i][k] A[k][j] ),
// one rounding from the host-precision source instead of the two of "convert, then merge", and
// the slot is written once.  The step hides under the host-to-device copy either way, so this
// kernel is written for clarity, not for the last percent: one wave per tile of 32 rows x 128
// columns, the delta tile from the matrix cores exactly as in the in-place merge (or, for the
// bit-reproducible mode, as one fused multiply-add chain in ascending k per element), sources
// read as 8- or 16-byte vectors where the piece covers whole aligned quads, element by element
// at the ragged ends of a piece (pieces are cut at element counts, not at row ends).
#include "lora_device.h"

namespace tidal {

template <int DT>
__device__ __forceinline__ float widen1(const void* src, int64_t idx) {
    if constexpr (DT == TIDAL_F32) return as_global((const float*)src)[idx];
    else return (float)as_global((const _Float16*)src)[idx];
}

template <int KS>
__device__ __forceinline__ void ordered_delta(const uint16_t* __restrict__ At, const uint16_t* __restrict__ Bp, int out,
                                              int in, int i0, int jl, int h, f32x16 (&acc)[4]) {
    constexpr int RP = 16 * KS;
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = (f32x16){0};
    for (int kb = 0; kb < RP; kb += 8) {
        float a8[4][8];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            int j = jl + c;
            j = j < in ? j : in - 1;
            const u32x4 v = as_global((const u32x4*)At)[at_group(j, kb >> 4, (kb >> 3) & 1, KS)];
            const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                a8[c][2 * e] = __uint_as_float(wds[e] << 16);
                a8[c][2 * e + 1] = __uint_as_float(wds[e] & 0xFFFF0000u);
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            int row = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
            row = row < out ? row : out - 1;
            const u32x4 bv = as_global((const u32x4*)Bp)[bp_group(row, kb >> 4, (kb >> 3) & 1, KS)];
            const uint32_t wds[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float b = (e & 1) ? __uint_as_float(wds[e >> 1] & 0xFFFF0000u) : __uint_as_float(wds[e >> 1] << 16);
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[c][v] = __builtin_fmaf(b, a8[c][e], acc[c][v]);
            }
        }
    }
}

template <int KS, int DT, bool ORDERED>
__global__ __launch_bounds__(256) void convert_merge_kernel(const FusedPiece p, int row_lo, int rowblocks, int strips,
                                                            int vec_ok) {
    constexpr int NT = 4;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t item = (int64_t)blockIdx.x * 4 + wave;
    if (item >= (int64_t)rowblocks * strips) return;
    const int rb = (int)(item / strips);
    const int strip = (int)(item - (int64_t)rb * strips);
    const int i0 = row_lo + rb * 32, j0 = strip * (32 * NT);
    const int n = lane & 31, h = lane >> 5;
    const int jl = j0 + NT * n;

    f32x16 acc[NT];
    if constexpr (ORDERED) {
        ordered_delta<KS>(p.At, p.Bp, p.out, p.in, i0, jl, h, acc);
    } else {
        bf16x8 bop[NT][KS], aop[KS];
        load_strip<NT, KS>(p.At, j0, lane, bop);              // 128-column strips: gathers from the 256-column packing
        {   // a piece may start at any row, so the 32 rows are not one packed block: gather, clamped to the last row
            int m = i0 + (lane & 31);
            m = m < p.out ? m : p.out - 1;
            const int64_t base = bp_group(m, 0, lane >> 5, KS);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) aop[ks] = as_global((const bf16x8*)p.Bp)[base + 64 * ks];
        }
        delta_tile<NT, KS>(aop, bop, acc);
    }
    const int64_t e_end = p.e0 + p.n;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
        const int64_t e = (int64_t)row * p.in + jl;
        if (row >= p.out || jl >= p.in) continue;
        if (vec_ok && jl + NT <= p.in && e >= p.e0 && e + NT <= e_end) {
            float w[4];
            if constexpr (DT == TIDAL_F32) {
                const f32x4 x = *as_global((const f32x4*)((const float*)p.src + (e - p.e0)));
                w[0] = x.x; w[1] = x.y; w[2] = x.z; w[3] = x.w;
            } else {
                typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                const h4 x = *as_global((const h4*)((const _Float16*)p.src + (e - p.e0)));
                w[0] = (float)x.x; w[1] = (float)x.y; w[2] = (float)x.z; w[3] = (float)x.w;
            }
            const f32x2 lo = {__builtin_fmaf(p.s, acc[0][v], w[0]), __builtin_fmaf(p.s, acc[1][v], w[1])};
            const f32x2 hi = {__builtin_fmaf(p.s, acc[2][v], w[2]), __builtin_fmaf(p.s, acc[3][v], w[3])};
            u32x2 o;
            o.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
            o.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
            *as_global((u32x2*)(p.slot + e)) = o;
        } else {
#pragma unroll
            for (int c = 0; c < NT; ++c) {
                if (jl + c < p.in && e + c >= p.e0 && e + c < e_end) {
                    const f32x2 r2 = {__builtin_fmaf(p.s, acc[c][v], widen1<DT>(p.src, e + c - p.e0)), 0.0f};
                    as_global(p.slot)[e + c] =
                        (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(r2, bf16x2)) & 0xFFFFu);
                }
            }
        }
    }
}

template <int KS, int DT>
static hipError_t launch_inst(const FusedPiece& p, bool ordered, hipStream_t stream) {
    const int64_t row_lo = p.e0 / p.in;
    const int64_t row_hi = (p.e0 + p.n + p.in - 1) / p.in;           // one past the last row touched
    const int rowblocks = (int)((row_hi - row_lo + 31) / 32);
    const int strips = (p.in + 127) / 128;
    const int64_t items = (int64_t)rowblocks * strips;
    if (items <= 0) return hipSuccess;
    if ((items + 3) / 4 > 0x7FFFFFF0) return hipErrorInvalidValue;
    const int vec_ok = (p.in % 4 == 0) && (p.e0 % 4 == 0);
    const dim3 grid((unsigned)((items + 3) / 4));
    if (ordered)
        hipLaunchKernelGGL((convert_merge_kernel<KS, DT, true>), grid, dim3(256), 0, stream, p, (int)row_lo, rowblocks,
                           strips, vec_ok);
    else
        hipLaunchKernelGGL((convert_merge_kernel<KS, DT, false>), grid, dim3(256), 0, stream, p, (int)row_lo, rowblocks,
                           strips, vec_ok);
    return hipGetLastError();
}

template <int DT>
static hipError_t launch_rank(const FusedPiece& p, bool ordered, hipStream_t stream) {
    switch (p.rp) {
        case 16: return launch_inst<1, DT>(p, ordered, stream);
        case 32: return launch_inst<2, DT>(p, ordered, stream);
        case 64: return launch_inst<4, DT>(p, ordered, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_convert_merge(const FusedPiece& p, bool ordered, hipStream_t stream) {
    if (p.n <= 0) return hipSuccess;
    if (p.out <= 0 || p.in <= 0 || p.e0 < 0 || p.e0 + p.n > (int64_t)p.out * p.in) return hipErrorInvalidValue;
    if (p.dtype == TIDAL_F32) return launch_rank<TIDAL_F32>(p, ordered, stream);
    if (p.dtype == TIDAL_F16) return launch_rank<TIDAL_F16>(p, ordered, stream);
    return hipErrorInvalidValue;                                      // bf16 sources are not staged
}

}  // namespace tidal
