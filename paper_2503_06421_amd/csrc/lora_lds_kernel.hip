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
    int m = i0 + (lane & 31);
    m = m < out ? m : out - 1;
    const uint16_t* p = Bp + (int64_t)m * (16 * KS) + 8 * (lane >> 5);
    bf16x8 aop[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) aop[ks] = *as_global((const bf16x8*)(p + 16 * ks));
#pragma unroll
    for (int T = 0; T < NT; ++T) {
        f32x16 c = {0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], strip[(T * KS + ks) * 64 + lane], c, 0, 0, 0);
        acc[T] = c;
    }
}

// The same with the tiles produced and consumed two at a time (32 live accumulator registers).
template <int NT, int KS>
__device__ __forceinline__ void delta_apply_lds(const uint16_t* __restrict__ Bp, int out, int i0, int lane,
                                                const bf16x8* strip, uint32_t (&w)[16][NT / 2], float s) {
    int m = i0 + (lane & 31);
    m = m < out ? m : out - 1;
    const uint16_t* p = Bp + (int64_t)m * (16 * KS) + 8 * (lane >> 5);
    bf16x8 aop[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) aop[ks] = *as_global((const bf16x8*)(p + 16 * ks));
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

template <int NT, int KS>
__device__ __forceinline__ void stage_strip(const uint16_t* __restrict__ At, int in, int j0, int lane, int wave,
                                            bf16x8* strip) {
    const int n = lane & 31, kg = lane >> 5;
    for (int p = wave; p < NT * KS; p += 4) {
        const int T = p / KS, ks = p - T * KS;
        int j = j0 + NT * n + T;
        j = j < in ? j : in - 1;
        strip[p * 64 + lane] = *as_global((const bf16x8*)(At + (int64_t)j * (16 * KS) + 16 * ks + 8 * kg));
    }
}

template <int NT, int KS0, int KS1>
__global__ __launch_bounds__(256) void lora_mfma_lds_kernel(const LoraBatch batch, int out,
                                                            int in, int strips, int rowblocks, int rcb,
                                                            int blocks_per_target, int total_blocks) {
    __shared__ bf16x8 strip_lds[(KS0 + KS1) * NT * 64];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int per_xcd = gridDim.x >> 3;
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= total_blocks) return;                        // whole workgroup leaves together
    const int target = L / blocks_per_target;
    const int item = L - target * blocks_per_target;
    const int rowchunk = item / strips;
    const int strip = item - rowchunk * strips;
    const int j0 = strip * (32 * NT);

    const LoraTargetDev d = batch.t[target];
    uint16_t* __restrict__ W = (uint16_t*)(batch.w_base + (size_t)d.w * kLoraUnit);
    const uint16_t* At_old = (const uint16_t*)(batch.old_base + (size_t)d.at_old * kLoraUnit);
    const uint16_t* Bp_old = (const uint16_t*)(batch.old_base + (size_t)d.bp_old * kLoraUnit);
    const uint16_t* At_new = (const uint16_t*)(batch.new_base + (size_t)d.at_new * kLoraUnit);
    const uint16_t* Bp_new = (const uint16_t*)(batch.new_base + (size_t)d.bp_new * kLoraUnit);
    if constexpr (KS0 > 0) stage_strip<NT, KS0>(At_old, in, j0, lane, wave, strip_lds);
    if constexpr (KS1 > 0) stage_strip<NT, KS1>(At_new, in, j0, lane, wave, strip_lds + KS0 * NT * 64);
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
            apply_tile<NT>(w, acc, d.s_old);
            delta_tile_lds<NT, KS1>(Bp_new, out, i0, lane, strip_lds + KS0 * NT * 64, acc);
            apply_tile<NT>(w, acc, d.s_new);
        }
        store_block<NT>(W, out, in, i0, jl, h, full, w);
    }
}

template <int NT, int KS0, int KS1>
static hipError_t launch_mfma_lds_inst(const LoraGroup& g, hipStream_t stream) {
    const int strips = (g.in + 32 * NT - 1) / (32 * NT);
    const int rowblocks = (g.out + 31) / 32;
    const int64_t tiles = (int64_t)strips * rowblocks * g.n_targets;
    // 32-row blocks per wave (measured, 64 and 128 slots of 4096^2, 40 of 5120^2 and 15 of the two
    // 13824-wide shapes): 16 for 64 -> 64, else 8; 4 and 2 where the row pitch is no power of two
    const bool pow2_pitch = (g.in & (g.in - 1)) == 0;
    int rc = (KS0 + KS1 >= 8) ? (pow2_pitch ? 16 : 4) : (pow2_pitch ? 8 : 2);
    const int64_t by_size = tiles / 4096;
    if (by_size < rc) rc = by_size < 1 ? 1 : (int)by_size;
    if (const char* e = tuning_knob("TIDAL_MFMA_RC")) {   // tuning builds only
        const int v = atoi(e);
        if (v >= 1 && v <= 1024) rc = v;
    }
    const int rcb = 4 * rc;
    const int rowchunks = (rowblocks + rcb - 1) / rcb;
    const int blocks_per_target = strips * rowchunks;
    const int64_t total = (int64_t)blocks_per_target * g.n_targets;
    if (total > 0x7FFFFFF0) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((total + 7) / 8 * 8);
    hipLaunchKernelGGL((lora_mfma_lds_kernel<NT, KS0, KS1>), dim3(grid), dim3(256), 0, stream, *g.batch, g.out,
                       g.in, strips, rowblocks, rcb, blocks_per_target, (int)total);
    return hipGetLastError();
}


bool lora_mfma_lds_available(int rp_old, int rp_new) {
    return (rp_old == 64 && rp_new >= 16) || (rp_new == 64 && rp_old >= 16);
}

hipError_t launch_lora_mfma_lds(const LoraGroup& g, hipStream_t stream) {
    if (g.rp_old == 64 && g.rp_new == 64) return launch_mfma_lds_inst<8, 4, 4>(g, stream);
    if (g.rp_old == 64 && g.rp_new == 32) return launch_mfma_lds_inst<8, 4, 2>(g, stream);
    if (g.rp_old == 64 && g.rp_new == 16) return launch_mfma_lds_inst<8, 4, 1>(g, stream);
    if (g.rp_old == 32 && g.rp_new == 64) return launch_mfma_lds_inst<8, 2, 4>(g, stream);
    if (g.rp_old == 16 && g.rp_new == 64) return launch_mfma_lds_inst<8, 1, 4>(g, stream);
    return hipErrorInvalidValue;
}

}  // namespace tidal
