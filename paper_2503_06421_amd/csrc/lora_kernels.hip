// In-place LoRA merge / unmerge / fused swap on template slots.  gfx950 only.
//
// The paper leaves the per-request (dynamic) part of initialisation -- attaching a LoRA
// adapter to the shared base weights -- to user code (Sec. 5.2, "Adaptive template state
// reusing"), and re-does only that part while a function is kept alive (Sec. 5.2,
// "Keep-alive of dynamic function").  Here that part is one streaming pass over every
// targeted W:
//     W[i][j] <- bf16( f32(W[i][j]) + s * sum_k f32(B[i][k]) * f32(A[k][j]) ),   s = +-alpha/r
// and a swap applies the old adapter with -s_old, rounds to bf16 in registers, then applies
// the new one with +s_new: one read and one write of W, bit-identical to two passes.
//
// The pass is bound by HBM traffic (4 bytes per W element), not by arithmetic, as long as
// the rank-r products do not run on the vector ALUs: at r = 16 the chain of fp32 FMAs alone
// needs about two thirds of the chip's (unpacked) fp32 rate at 70 % of HBM bandwidth, at
// r = 64 it needs 2.6x more than exists.  So two kernels:
//
//  * lora_mfma_kernel (default): each wave owns a column strip of W and walks down its rows
//    in 32-row blocks.  The 32 x (32*NT) tile of sum_k B A is produced by NT
//    v_mfma_f32_32x32x16_bf16 per 16 ranks straight into registers -- there is no separate
//    GEMM and the delta never exists in memory.  The strip of A stays in registers for the
//    whole walk (column-strip stationary), the 32 rows of B are one 16-byte load per lane,
//    and the MFMA output layout is matched to memory by choosing which column feeds which
//    MFMA column index: lane n of tile T owns column NT*n + T, so a lane holds NT adjacent
//    columns of a row and a wave-wide access covers two full rows of 64*NT contiguous bytes.
//    fp32 accumulation order inside the MFMA is the hardware's.
//
//  * lora_ordered_kernel (TIDAL_FLAG_ORDERED_ACCUM): 64 x 256 tiles, A and B rank tiles
//    staged in LDS as fp32, 128-bit accesses to W, and the sum taken as one fused
//    multiply-add chain in ascending k per element -- reproducible bit for bit against a
//    sequential definition; VALU-bound from r = 16 up.
#include "lora_device.h"

namespace tidal {

// FORK: the result goes to a separate destination (old_base + at_old, which are free because a
// fork never unmerges: KS0 == 0) and W itself, the template's pristine slot, is only read.
// PAIR: the delta tiles are produced and consumed two at a time (32 live accumulator registers
// instead of 128).  Instantiations whose registers then allow two waves per SIMD without spilling
// ask for them (two_waves_fit).
template <int NT, int KS0, int KS1, bool FORK = false, bool PAIR = false>
__global__ __launch_bounds__(256, (PAIR && two_waves_fit(KS0, KS1)) ? 2 : 1) void lora_mfma_kernel(
    const LoraBatch batch, int out, int in, int strips, int rowblocks, int rc, int blocks_per_target, int total_blocks) {
    static_assert(!FORK || KS0 == 0, "a fork starts from the pristine template: nothing to unmerge");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroups are dealt round-robin to the 8 XCDs; undo that so that each XCD walks a
    // contiguous range of (target, row chunk, strip) and its L2 sees each A strip and each
    // B row block once.  gridDim.x is a multiple of 8.
    const int per_xcd = gridDim.x >> 3;
    const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (L >= total_blocks) return;
    const int target = L / blocks_per_target;
    const int item = (L - target * blocks_per_target) * 4 + wave;
    const int rowchunks = (rowblocks + rc - 1) / rc;
    if (item >= strips * rowchunks) return;
    const int rowchunk = item / strips;
    const int strip = item - rowchunk * strips;
    const int j0 = strip * (32 * NT);

    const LoraTargetDev d = batch.t[target];
    uint16_t* __restrict__ W = (uint16_t*)(batch.w_base + (size_t)d.w * kLoraUnit);
    const uint16_t* At_old = (const uint16_t*)(batch.old_base + (size_t)d.at_old * kLoraUnit);
    const uint16_t* Bp_old = (const uint16_t*)(batch.old_base + (size_t)d.bp_old * kLoraUnit);
    const uint16_t* At_new = (const uint16_t*)(batch.new_base + (size_t)d.at_new * kLoraUnit);
    const uint16_t* Bp_new = (const uint16_t*)(batch.new_base + (size_t)d.bp_new * kLoraUnit);

    bf16x8 bop0[NT][KS0 ? KS0 : 1];
    bf16x8 bop1[NT][KS1 ? KS1 : 1];
    load_strip<NT, KS0>(At_old, j0, lane, bop0);
    load_strip<NT, KS1>(At_new, j0, lane, bop1);

    const int n = lane & 31, h = lane >> 5;
    const int jl = j0 + NT * n;                              // lane's first column
    const bool strip_full = (j0 + 32 * NT <= in) && (in % NT == 0);
    const int rb_end = (rowchunk + 1) * rc < rowblocks ? (rowchunk + 1) * rc : rowblocks;

    // One block of loads per wave is in flight at a time.  Requesting the next 32-row block early
    // (software prefetch, a second set of W registers) was measured: 2-3 % slower on power-of-two
    // pitches, 1-2 % faster on the others for merges of up to 32 ranks at 2 blocks per wave, nothing
    // at 64 ranks -- not worth a second set of instantiations.
    for (int rb = rowchunk * rc; rb < rb_end; ++rb) {
        const int i0 = rb * 32;
        const bool full = strip_full && (i0 + 32 <= out);
        uint32_t w[16][NT / 2];
        load_block<NT>(W, out, in, i0, jl, h, full, w);
        if constexpr (PAIR) {
            delta_apply<NT, KS0>(Bp_old, i0, lane, bop0, w, d.s_old);
            delta_apply<NT, KS1>(Bp_new, i0, lane, bop1, w, d.s_new);
        } else {
            f32x16 acc[NT];
            if constexpr (KS0 > 0) {
                bf16x8 aop[KS0];
                load_b_rows<KS0>(Bp_old, i0, lane, aop);
                delta_tile<NT, KS0>(aop, bop0, acc);
                apply_tile<NT>(w, acc, d.s_old);
            }
            if constexpr (KS1 > 0) {
                bf16x8 aop[KS1];
                load_b_rows<KS1>(Bp_new, i0, lane, aop);
                delta_tile<NT, KS1>(aop, bop1, acc);
                apply_tile<NT>(w, acc, d.s_new);
            }
        }
        store_block<NT>(FORK ? (uint16_t*)(batch.old_base + (size_t)d.at_old * kLoraUnit) : W, out, in, i0, jl, h,
                        full, w);
    }
}

// Launch of one instantiation with the walk length and grid the plan gives.
template <int KS0, int KS1, bool FORK, bool PAIR>
static hipError_t launch_inst(const LoraGroup& g, const LoraLaunchPlan& p, hipStream_t stream) {
    if (p.total_blocks <= 0 || p.total_blocks > 0x7FFFFFF0) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)((p.total_blocks + 7) / 8 * 8);
    hipLaunchKernelGGL((lora_mfma_kernel<8, KS0, KS1, FORK, PAIR>), dim3(grid), dim3(256), 0, stream, *g.batch, g.out,
                       g.in, p.strips, p.rowblocks, p.rc, p.blocks_per_target, (int)p.total_blocks);
    return hipGetLastError();
}

template <int KS0, int KS1>
static hipError_t launch_variant(const LoraGroup& g, const LoraLaunchPlan& p, hipStream_t stream) {
    if constexpr (KS0 + KS1 == 0) {
        return hipSuccess;
    } else {
        if (p.fork) {
            if constexpr (KS0 == 0)
                return p.pair ? launch_inst<0, KS1, true, true>(g, p, stream) : launch_inst<0, KS1, true, false>(g, p, stream);
            else
                return hipErrorInvalidValue;
        }
        return p.pair ? launch_inst<KS0, KS1, false, true>(g, p, stream) : launch_inst<KS0, KS1, false, false>(g, p, stream);
    }
}

template <int KS0>
static hipError_t launch_new(const LoraGroup& g, const LoraLaunchPlan& p, hipStream_t stream) {
    switch (p.ks_new) {
        case 0: return launch_variant<KS0, 0>(g, p, stream);
        case 1: return launch_variant<KS0, 1>(g, p, stream);
        case 2: return launch_variant<KS0, 2>(g, p, stream);
        case 4: return launch_variant<KS0, 4>(g, p, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_lora_mfma(const LoraGroup& g, const LoraLaunchPlan& p, hipStream_t stream) {
    if (p.kind == kLoraNone) return hipSuccess;
    if (p.kind == kLoraMfmaLds) return launch_lora_mfma_lds(g, p, stream);
    if (p.kind != kLoraMfmaReg) return hipErrorInvalidValue;
    switch (p.ks_old) {
        case 0: return launch_new<0>(g, p, stream);
        case 1: return launch_new<1>(g, p, stream);
        case 2: return launch_new<2>(g, p, stream);
        case 4: return launch_new<4>(g, p, stream);
    }
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------
// Ordered-accumulation kernel (vector ALUs, LDS-staged rank tiles)
// ---------------------------------------------------------------------------------------
constexpr int kOrdRows = 64, kOrdCols = 256, kOrdK = 16;

// Stage ranks [k0, k0+16) of the A strip (as Atile[k][col]) and of the B rows (as
// Btile[k][row]) into LDS as fp32.  The packed layouts are zero padded to a multiple of 16
// ranks, so no k bound is needed here.
__device__ __forceinline__ void stage_rank_tiles(const uint16_t* __restrict__ At, const uint16_t* __restrict__ Bp,
                                                 int rp, int out, int in, int i0, int j0, int k0,
                                                 float* Atile, float* Btile) {
    const int tid = threadIdx.x;
    const int KS = rp >> 4, ks = k0 >> 4;
    {   // 256 columns x 16 ranks: one column per thread, two 16-byte groups (columns past `in` are zero padding)
        const TIDAL_GLOBAL u32x4* g = as_global((const u32x4*)At);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            u32x4 x = g[at_group(j0 + tid, ks, q, KS)];
            const uint32_t wds[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                Atile[(8 * q + 2 * e) * kOrdCols + tid] = __uint_as_float(wds[e] << 16);
                Atile[(8 * q + 2 * e + 1) * kOrdCols + tid] = __uint_as_float(wds[e] & 0xFFFF0000u);
            }
        }
    }
    if (tid < 128) {   // 64 rows x 16 ranks: one 16-byte group per thread
        const int row = tid & 63, q = tid >> 6;
        int i = i0 + row;
        i = i < out ? i : out - 1;
        u32x4 x = as_global((const u32x4*)Bp)[bp_group(i, ks, q, KS)];
        const uint32_t wds[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            Btile[(8 * q + 2 * e) * kOrdRows + row] = __uint_as_float(wds[e] << 16);
            Btile[(8 * q + 2 * e + 1) * kOrdRows + row] = __uint_as_float(wds[e] & 0xFFFF0000u);
        }
    }
}

__device__ __forceinline__ void ordered_phase(const uint16_t* __restrict__ At, const uint16_t* __restrict__ Bp,
                                              int r, int rp, float s, int out, int in, int i0, int j0,
                                              float* Atile, float* Btile, uint32_t (&w)[8][4]) {
    const int cg = threadIdx.x & 31, rg = threadIdx.x >> 5;
    float acc[8][8];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) acc[a][b] = 0.0f;
    for (int k0 = 0; k0 < r; k0 += kOrdK) {
        __syncthreads();
        stage_rank_tiles(At, Bp, rp, out, in, i0, j0, k0, Atile, Btile);
        __syncthreads();
        const int kend = (r - k0) < kOrdK ? (r - k0) : kOrdK;
        for (int k = 0; k < kend; ++k) {
            const f32x4 a_lo = *(const f32x4*)(Atile + k * kOrdCols + 8 * cg);
            const f32x4 a_hi = *(const f32x4*)(Atile + k * kOrdCols + 8 * cg + 4);
            const f32x4 b_lo = *(const f32x4*)(Btile + k * kOrdRows + 8 * rg);
            const f32x4 b_hi = *(const f32x4*)(Btile + k * kOrdRows + 8 * rg + 4);
            const float a8[8] = {a_lo.x, a_lo.y, a_lo.z, a_lo.w, a_hi.x, a_hi.y, a_hi.z, a_hi.w};
            const float b8[8] = {b_lo.x, b_lo.y, b_lo.z, b_lo.w, b_hi.x, b_hi.y, b_hi.z, b_hi.w};
#pragma unroll
            for (int rr = 0; rr < 8; ++rr)
#pragma unroll
                for (int cc = 0; cc < 8; ++cc) acc[rr][cc] = __builtin_fmaf(b8[rr], a8[cc], acc[rr][cc]);
        }
    }
#pragma unroll
    for (int rr = 0; rr < 8; ++rr)
#pragma unroll
        for (int p = 0; p < 4; ++p) w[rr][p] = rmw2(w[rr][p], acc[rr][2 * p], acc[rr][2 * p + 1], s);
}

__global__ __launch_bounds__(256) void lora_ordered_kernel(const LoraBatch batch, int out,
                                                           int in, int r_old, int rp_old, int r_new,
                                                           int rp_new, int col_tiles, int tiles_per_target,
                                                           int fork) {
    __shared__ __attribute__((aligned(16))) float Atile[kOrdK * kOrdCols];
    __shared__ __attribute__((aligned(16))) float Btile[kOrdK * kOrdRows];
    const int target = blockIdx.x / tiles_per_target;
    const int tile = blockIdx.x - target * tiles_per_target;
    const int i0 = (tile / col_tiles) * kOrdRows;
    const int j0 = (tile % col_tiles) * kOrdCols;
    const LoraTargetDev d = batch.t[target];
    uint16_t* __restrict__ W = (uint16_t*)(batch.w_base + (size_t)d.w * kLoraUnit);
    const uint16_t* At_old = (const uint16_t*)(batch.old_base + (size_t)d.at_old * kLoraUnit);
    const uint16_t* Bp_old = (const uint16_t*)(batch.old_base + (size_t)d.bp_old * kLoraUnit);
    const uint16_t* At_new = (const uint16_t*)(batch.new_base + (size_t)d.at_new * kLoraUnit);
    const uint16_t* Bp_new = (const uint16_t*)(batch.new_base + (size_t)d.bp_new * kLoraUnit);
    const int cg = threadIdx.x & 31, rg = threadIdx.x >> 5;
    const int jl = j0 + 8 * cg;
    const bool vec_ok = (in % 8 == 0) && (jl + 8 <= in);

    uint32_t w[8][4];
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const int row = i0 + 8 * rg + rr;
        if (vec_ok && row < out) {
            u32x4 x = *as_global((const u32x4*)(W + (int64_t)row * in + jl));
            w[rr][0] = x.x; w[rr][1] = x.y; w[rr][2] = x.z; w[rr][3] = x.w;
        } else {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                uint32_t lo = 0, hi = 0;
                if (row < out && jl + 2 * p < in) lo = as_global(W)[(int64_t)row * in + jl + 2 * p];
                if (row < out && jl + 2 * p + 1 < in) hi = as_global(W)[(int64_t)row * in + jl + 2 * p + 1];
                w[rr][p] = lo | (hi << 16);
            }
        }
    }
    uint16_t* __restrict__ Wd = fork ? (uint16_t*)(batch.old_base + (size_t)d.at_old * kLoraUnit) : W;
    if (rp_old > 0) ordered_phase(At_old, Bp_old, r_old, rp_old, d.s_old, out, in, i0, j0, Atile, Btile, w);
    if (rp_new > 0) ordered_phase(At_new, Bp_new, r_new, rp_new, d.s_new, out, in, i0, j0, Atile, Btile, w);
#pragma unroll
    for (int rr = 0; rr < 8; ++rr) {
        const int row = i0 + 8 * rg + rr;
        if (vec_ok && row < out) {
            u32x4 x;
            x.x = w[rr][0]; x.y = w[rr][1]; x.z = w[rr][2]; x.w = w[rr][3];
            *as_global((u32x4*)(Wd + (int64_t)row * in + jl)) = x;
        } else {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if (row < out && jl + 2 * p < in) as_global(Wd)[(int64_t)row * in + jl + 2 * p] = (uint16_t)(w[rr][p] & 0xFFFFu);
                if (row < out && jl + 2 * p + 1 < in) as_global(Wd)[(int64_t)row * in + jl + 2 * p + 1] = (uint16_t)(w[rr][p] >> 16);
            }
        }
    }
}

hipError_t launch_lora_ordered(const LoraGroup& g, hipStream_t stream) {
    if (g.n_targets <= 0 || g.out <= 0 || g.in <= 0) return hipSuccess;
    if (g.rp_old == 0 && g.rp_new == 0) return hipSuccess;
    const int col_tiles = (g.in + kOrdCols - 1) / kOrdCols;
    const int row_tiles = (g.out + kOrdRows - 1) / kOrdRows;
    const int64_t tiles_per_target = (int64_t)col_tiles * row_tiles;
    const int64_t total = tiles_per_target * g.n_targets;
    if (total > 0x7FFFFFF0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(lora_ordered_kernel, dim3((unsigned)total), dim3(256), 0, stream, *g.batch, g.out, g.in,
                       g.r_old, g.rp_old, g.r_new, g.rp_new, col_tiles, (int)tiles_per_target, g.fork ? 1 : 0);
    return hipGetLastError();
}

}  // namespace tidal
