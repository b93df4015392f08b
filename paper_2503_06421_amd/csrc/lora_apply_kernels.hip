// Unmerged LoRA adapters applied to activations of a mixed batch.  gfx950 only.
//
// The paper's dynamic function keeps each request's adapter as separate weights beside the shared
// base model (Sec. 3, programming interface; Sec. 5.2, adaptive template state reusing), so that
// requests with different adapters can share a batch.  For the tokens t of one request
//     u[t] = bf16( A x[t] ),      y[t] <- bf16( y[t] + s * B u[t] ),      s = alpha / r
// with fp32 accumulation.  Tokens are cut into tiles of up to 32 rows that share an adapter; both
// steps run on the matrix cores (v_mfma_f32_32x32x16_bf16) with the token rows as the M index:
//
//  * apply_shrink_kernel: one workgroup of 8 waves per tile.  The contraction runs over the whole
//    input width, so the waves split it: wave w takes the 64-column groups w, w+8, ... and a lane
//    reads 64 contiguous bytes of its x row and of its A row per group (both operands use the same
//    column permutation, which a sum does not care about), giving full 128-byte lines per row.
//    The 8 partial 32 x rp tiles meet in LDS and are added in wave order, so the result does not
//    depend on scheduling.  u goes to the caller's workspace as rows x rp bf16.
//
//  * apply_expand_kernel: the same register tiling as the in-place merge with y in the place of W
//    (rows = tokens, columns = out), B's rows as the stationary strip and u as the per-row factor:
//    a lane owns 8 adjacent outputs of 16 token rows, 128-bit accesses to y.
//
// HBM traffic: x once, y read and written once, the factors once per adapter (L2 serves tiles that
// share one), u is a few KB per tile.
#include "lora_device.h"

namespace tidal {

constexpr int kShrinkWaves = 8;

__device__ __forceinline__ bf16x8 zero8() {
    const u32x4 z = {0u, 0u, 0u, 0u};
    return __builtin_bit_cast(bf16x8, z);
}

template <bool TWO>
__device__ __forceinline__ void shrink_accumulate(const uint16_t* __restrict__ xrow, const uint16_t* __restrict__ a0,
                                                  const uint16_t* __restrict__ a1, bool v0, bool v1, int in, int kg,
                                                  int wave, f32x16& c0, f32x16& c1) {
    const int groups = (in + 63) >> 6;
    for (int g = wave; g < groups; g += kShrinkWaves) {
        const int jb = g * 64 + 32 * kg;                        // lane's first column in this group
        bf16x8 xv[4], av0[4], av1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool ok = jb + 8 * q + 8 <= in;               // in is a multiple of 8
            const int j = ok ? jb + 8 * q : 0;
            const bf16x8 xl = *as_global((const bf16x8*)(xrow + j));
            const bf16x8 al0 = *as_global((const bf16x8*)(a0 + j));
            xv[q] = ok ? xl : zero8();
            av0[q] = (ok && v0) ? al0 : zero8();
            if constexpr (TWO) {
                const bf16x8 al1 = *as_global((const bf16x8*)(a1 + j));
                av1[q] = (ok && v1) ? al1 : zero8();
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xv[q], av0[q], c0, 0, 0, 0);
            if constexpr (TWO) c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xv[q], av1[q], c1, 0, 0, 0);
        }
    }
}

__global__ __launch_bounds__(64 * kShrinkWaves) void apply_shrink_kernel(const ApplyBatch batch, int in) {
    __shared__ float part[kShrinkWaves][2][32][32];             // 64 KB: [wave][rank tile][token][rank]
    const ApplyTile tl = batch.tile[blockIdx.x];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, kg = lane >> 5;
    // A operand (M x K): token rows of x; rows past the tile repeat its last row and are dropped
    const int tok = tl.t0 + (n < tl.rows ? n : tl.rows - 1);
    const uint16_t* xrow = batch.x + (int64_t)tok * in;
    // B operand (K x N): rank rows of A; ranks past r read row 0 and are zeroed
    const bool v0 = n < tl.r, v1 = n + 32 < tl.r;
    const uint16_t* a0 = tl.Ar + (int64_t)(v0 ? n : 0) * in;
    const uint16_t* a1 = tl.Ar + (int64_t)(v1 ? n + 32 : 0) * in;
    const bool two = tl.rp > 32;

    f32x16 c0 = {0}, c1 = {0};
    if (two) shrink_accumulate<true>(xrow, a0, a1, v0, v1, in, kg, wave, c0, c1);
    else shrink_accumulate<false>(xrow, a0, a1, v0, v1, in, kg, wave, c0, c1);

    // C layout: lane holds rank column n of token rows 8*(v/4) + 4*kg + v%4
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = 8 * (v >> 2) + 4 * kg + (v & 3);
        part[wave][0][row][n] = c0[v];
        if (two) part[wave][1][row][n] = c1[v];
    }
    __syncthreads();
    uint32_t* u = (uint32_t*)(batch.u + (int64_t)tl.t0 * kApplyRankStride);
    const int pairs_per_row = tl.rp >> 1;
    const int pairs = tl.rows * pairs_per_row;
    for (int e = threadIdx.x; e < pairs; e += 64 * kShrinkWaves) {
        const int row = e / pairs_per_row;
        const int k = 2 * (e - row * pairs_per_row);
        float lo = 0.0f, hi = 0.0f;
#pragma unroll
        for (int w = 0; w < kShrinkWaves; ++w) {                // fixed order: reproducible
            lo += part[w][k >> 5][row][k & 31];
            hi += part[w][k >> 5][row][(k & 31) + 1];
        }
        const f32x2 r2 = {lo, hi};
        as_global(u)[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(r2, bf16x2));
    }
}

hipError_t launch_apply_shrink(const ApplyBatch& b, int n_tiles, int in, hipStream_t stream) {
    if (n_tiles <= 0) return hipSuccess;
    if (n_tiles > kMaxApplyTiles || in <= 0 || in % 8) return hipErrorInvalidValue;
    hipLaunchKernelGGL(apply_shrink_kernel, dim3((unsigned)n_tiles), dim3(64 * kShrinkWaves), 0, stream, b, in);
    return hipGetLastError();
}

template <int KS>
__device__ __forceinline__ void expand_tile(const ApplyBatch& batch, const ApplyTile& tl, int out, int j0, int lane) {
    constexpr int NT = 8;
    bf16x8 bop[NT][KS];
    load_strip<NT, KS>(tl.Bp, out, j0, lane, bop);              // rows of B for the lane's 8 outputs
    const uint16_t* u = batch.u + (int64_t)tl.t0 * kApplyRankStride;
    f32x16 acc[NT];
    delta_tile<NT, KS>(u, tl.rows, 0, lane, bop, acc);
    const int n = lane & 31, h = lane >> 5;
    const int jl = j0 + NT * n;
    uint16_t* y = batch.y + (int64_t)tl.t0 * out;
    const bool full = (tl.rows == 32) && (j0 + 32 * NT <= out);
    uint32_t w[16][NT / 2];
    load_block<NT>(y, tl.rows, out, 0, jl, h, full, w);
    apply_tile<NT>(w, acc, tl.s);
    store_block<NT>(y, tl.rows, out, 0, jl, h, full, w);
}

__global__ __launch_bounds__(256) void apply_expand_kernel(const ApplyBatch batch, int n_tiles, int out, int strips) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int item = blockIdx.x * 4 + wave;
    if (item >= n_tiles * strips) return;
    // neighbouring waves take neighbouring tiles of one strip: they share the rows of B
    const int strip = item / n_tiles;
    const int tile = item - strip * n_tiles;
    const ApplyTile tl = batch.tile[tile];
    const int j0 = strip * 256;
    switch (tl.rp) {
        case 16: expand_tile<1>(batch, tl, out, j0, lane); break;
        case 32: expand_tile<2>(batch, tl, out, j0, lane); break;
        case 64: expand_tile<4>(batch, tl, out, j0, lane); break;
        default: break;
    }
}

hipError_t launch_apply_expand(const ApplyBatch& b, int n_tiles, int out, hipStream_t stream) {
    if (n_tiles <= 0) return hipSuccess;
    if (n_tiles > kMaxApplyTiles || out <= 0 || out % 8) return hipErrorInvalidValue;
    const int strips = (out + 255) / 256;
    const int64_t items = (int64_t)n_tiles * strips;
    hipLaunchKernelGGL(apply_expand_kernel, dim3((unsigned)((items + 3) / 4)), dim3(256), 0, stream, b, n_tiles, out,
                       strips);
    return hipGetLastError();
}

}  // namespace tidal
