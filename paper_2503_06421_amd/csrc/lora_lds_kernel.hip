// LoRA fused swap where one adapter has 64 ranks: A strips staged in LDS.  gfx950 only.
//
// This file is compiled with -mllvm -amdgpu-mfma-vgpr-form: the MFMA results land in ordinary
// VGPRs, which saves one accumulator-read instruction per element and, here, lets two or three
// waves share a SIMD.  The other LoRA kernels are faster with the accumulators in AGPRs and stay
// in their own translation unit.
#include "lora_device.h"

namespace tidal {

// Variant for large ranks.  With 64 + 64 ranks the A strips of both adapters would need 256
// VGPRs per lane; instead the four waves of a workgroup share ONE column strip, stage its A
// operands once in LDS -- already in MFMA operand order, so every later read is a linear,
// conflict-free 16-byte-per-lane ds_read -- and take interleaved 32-row blocks of the same
// row range.  Registers then hold only the accumulators and W, which buys a second or third
// wave per SIMD exactly where the arithmetic per block is largest.
template <int NT, int KS>
__device__ __forceinline__ void delta_tile_lds(const uint16_t* __restrict__ Bp, int out, int i0, int lane,
                                               const bf16x8* strip, f32x16 (&acc)[NT]) {
    if constexpr (KS > 0) {
        bf16x8 aop[KS];
        load_b_rows<KS>(Bp, i0, lane, aop);
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            f32x16 c = {0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], strip[(T * KS + ks) * 64 + lane], c, 0, 0, 0);
            acc[T] = c;
        }
    }
}

// The same with the tiles produced and consumed two at a time (32 live accumulator registers).
template <int NT, int KS>
__device__ __forceinline__ void delta_apply_lds(const uint16_t* __restrict__ Bp, int out, int i0, int lane,
                                                const bf16x8* strip, uint32_t (&w)[16][NT / 2], float s) {
    if constexpr (KS > 0) {
        bf16x8 aop[KS];
        load_b_rows<KS>(Bp, i0, lane, aop);
#pragma unroll
        for (int q = 0; q < NT / 2; ++q) {
            f32x16 c0 = {0}, c1 = {0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], strip[((2 * q) * KS + ks) * 64 + lane], c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], strip[((2 * q + 1) * KS + ks) * 64 + lane], c1, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) w[v][q] = rmw2(w[v][q], c0[v], c1[v], s);
        }
    }
}

// The packed A of a strip is already in MFMA operand order: staging it is a linear copy of
// NT * KS kilobytes, one per (tile, 16 ranks).
template <int NT, int KS>
__device__ __forceinline__ void stage_strip(const uint16_t* __restrict__ At, int j0, int lane, int wave, bf16x8* strip) {
    const TIDAL_GLOBAL bf16x8* g = as_global((const bf16x8*)At) + (int64_t)(j0 >> 8) * (8 * KS * 64);
    for (int p = wave; p < NT * KS; p += 4) strip[p * 64 + lane] = g[p * 64 + lane];
}

template <int NT, int KS0, int KS1>
__global__ __launch_bounds__(256) void lora_mfma_lds_kernel(const LoraBatch batch, int out,
                                                            int in, int strips, int rowblocks, int rcb,
                                                            int blocks_per_target, int total_blocks, int order) {
    __shared__ bf16x8 strip_lds[(KS0 + KS1) * NT * 64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // order bit 1: no XCD remap (neighbouring workgroups land on different XCDs); bit 0: walk a
    // slot strip by strip (neighbouring workgroups share an A strip) instead of row chunk by row chunk
    const int per_xcd = gridDim.x >> 3;
    const int L = (order & 2) ? (int)blockIdx.x : (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= total_blocks) return;                        // whole workgroup leaves together
    const int target = L / blocks_per_target;
    const int item = L - target * blocks_per_target;
    const int rowchunks = blocks_per_target / strips;
    const int rowchunk = (order & 1) ? item % rowchunks : item / strips;
    const int strip = (order & 1) ? item / rowchunks : item - rowchunk * strips;
    const int j0 = strip * (32 * NT);

    const LoraTargetDev d = batch.t[target];
    uint16_t* __restrict__ W = (uint16_t*)(batch.w_base + (size_t)d.w * kLoraUnit);
    const uint16_t* At_old = (const uint16_t*)(batch.old_base + (size_t)d.at_old * kLoraUnit);
    const uint16_t* Bp_old = (const uint16_t*)(batch.old_base + (size_t)d.bp_old * kLoraUnit);
    const uint16_t* At_new = (const uint16_t*)(batch.new_base + (size_t)d.at_new * kLoraUnit);
    const uint16_t* Bp_new = (const uint16_t*)(batch.new_base + (size_t)d.bp_new * kLoraUnit);
    if constexpr (KS0 > 0) stage_strip<NT, KS0>(At_old, j0, lane, wave, strip_lds);
    if constexpr (KS1 > 0) stage_strip<NT, KS1>(At_new, j0, lane, wave, strip_lds + KS0 * NT * 64);
    __syncthreads();

    const int n = lane & 31, h = lane >> 5;
    const int jl = j0 + NT * n;
    const bool strip_full = (j0 + 32 * NT <= in) && (in % NT == 0);
    const int rb_end = (rowchunk + 1) * rcb < rowblocks ? (rowchunk + 1) * rcb : rowblocks;
    for (int rb = rowchunk * rcb + wave; rb < rb_end; rb += 4) {
        const int i0 = rb * 32;
        const bool full = strip_full && (i0 + 32 <= out);
        uint32_t w[16][NT / 2];
        load_block<NT>(W, out, in, i0, jl, h, full, w);
        // Tiles two at a time (three waves per SIMD at 64 -> 16/32, measured 6.5 against 5.4-5.8 TB/s
        // with all eight live); 64 -> 64 is the exception, 2 % faster with all eight.
        if constexpr (KS0 + KS1 < 8) {
            delta_apply_lds<NT, KS0>(Bp_old, out, i0, lane, strip_lds, w, d.s_old);
            delta_apply_lds<NT, KS1>(Bp_new, out, i0, lane, strip_lds + KS0 * NT * 64, w, d.s_new);
        } else {
            f32x16 acc[NT];
            delta_tile_lds<NT, KS0>(Bp_old, out, i0, lane, strip_lds, acc);
            if constexpr (KS0 > 0) apply_tile<NT>(w, acc, d.s_old);
            delta_tile_lds<NT, KS1>(Bp_new, out, i0, lane, strip_lds + KS0 * NT * 64, acc);
            if constexpr (KS1 > 0) apply_tile<NT>(w, acc, d.s_new);
        }
        store_block<NT>(W, out, in, i0, jl, h, full, w);
    }
}

template <int KS0, int KS1>
static hipError_t launch_lds_inst(const LoraGroup& g, const LoraLaunchPlan& p, hipStream_t stream) {
    if (p.total_blocks <= 0 || p.total_blocks > 0x7FFFFFF0) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((p.total_blocks + 7) / 8 * 8);
    const TuningKnobs knobs = tuning_knobs();              // all -1 outside tuning builds
    const int order = knobs.mfma_order > 0 ? knobs.mfma_order : 0;
    unsigned dyn = 0;
    if (knobs.mfma_dynlds > 0) {
        dyn = (unsigned)knobs.mfma_dynlds;
        hipError_t e = hipFuncSetAttribute((const void*)lora_mfma_lds_kernel<8, KS0, KS1>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((lora_mfma_lds_kernel<8, KS0, KS1>), dim3(grid), dim3(256), dyn, stream, *g.batch, g.out, g.in,
                       p.strips, p.rowblocks, 4 * p.rc, p.blocks_per_target, (int)p.total_blocks, order);
    return hipGetLastError();
}

hipError_t launch_lora_mfma_lds(const LoraGroup& g, const LoraLaunchPlan& p, hipStream_t stream) {
    if (p.kind != kLoraMfmaLds || p.fork) return hipErrorInvalidValue;
    switch (p.ks_old * 8 + p.ks_new) {
        case 4 * 8 + 4: return launch_lds_inst<4, 4>(g, p, stream);
        case 4 * 8 + 2: return launch_lds_inst<4, 2>(g, p, stream);
        case 4 * 8 + 1: return launch_lds_inst<4, 1>(g, p, stream);
        case 2 * 8 + 4: return launch_lds_inst<2, 4>(g, p, stream);
        case 1 * 8 + 4: return launch_lds_inst<1, 4>(g, p, stream);
        case 0 * 8 + 4: return launch_lds_inst<0, 4>(g, p, stream);
        case 0 * 8 + 2: return launch_lds_inst<0, 2>(g, p, stream);
        case 0 * 8 + 1: return launch_lds_inst<0, 1>(g, p, stream);
        case 4 * 8 + 0: return launch_lds_inst<4, 0>(g, p, stream);
        case 2 * 8 + 0: return launch_lds_inst<2, 0>(g, p, stream);
        case 1 * 8 + 0: return launch_lds_inst<1, 0>(g, p, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace tidal
