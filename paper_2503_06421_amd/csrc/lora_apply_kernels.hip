// Unmerged LoRA adapters applied to activations of a mixed batch.  gfx950 only.
//
// The paper's dynamic function keeps each request's adapter as separate weights beside the shared
// base model (Sec. 3, programming interface; Sec. 5.2, adaptive template state reusing), so that
// requests with different adapters can share a batch.  For the tokens t of one request
//     u[t] = bf16( A x[t] ),      y[t] <- bf16( y[t] + s * B u[t] ),      s = alpha / r
// with fp32 accumulation.  A batch is a list of segments (runs of token rows with one adapter).
//
// Segments of more than 4 tokens (prompts) run on the matrix cores, shorter ones (decode steps),
// where nearly all traffic is the factors themselves, on the vector ALUs:
//
//  * apply_shrink_kernel: one workgroup of 4 waves per tile of 32 tokens.  The contraction runs
//    over the whole input width, so the waves split it by groups of 64 columns.  The MFMA operand
//    layout puts consecutive lanes on consecutive rows, which as a global access pattern touches
//    32 cache lines per instruction for 16 useful bytes each; instead a wave fetches its group of
//    x (32 rows x 128 bytes) and of A (r rows x 128 bytes) with full-line accesses (8 lanes per
//    row), parks it in a private piece of LDS and reads the operands back from there in MFMA
//    order (row pitch 144 bytes: conflict-free 128-bit reads).  Only that wave touches its piece,
//    so the loop has no workgroup barrier; the next group's global loads are in flight while the
//    current one is multiplied.  The four partial 32 x rp tiles meet in LDS at the end and are
//    added in wave order, so the result does not depend on scheduling.  u goes to the caller's
//    workspace as rows x rp bf16 with zeros in the padded ranks.
//
//  * apply_expand_kernel: the register tiling of the
//    in-place merge with y in the place of W (rows = tokens, columns = out): B's rows for 256
//    outputs are the stationary strip, a wave walks down one to four 32-token tiles of one
//    segment (fewer when the batch is small, so that every CU has work), u is the per-row factor, a lane owns 8 adjacent outputs of 16 token rows and
//    accesses y with 128-bit vectors.
//
//  * apply_shrink_short_kernel: one wave per rank row, lanes along the input width (1 KB per
//    wave-wide load), one cross-lane reduction per token at the end.
//
//  * apply_expand_short_kernel: one lane per output.  The
//    lane's row of B is 32..128 contiguous bytes and neighbouring lanes read neighbouring rows,
//    so the factors -- nearly all of the traffic here -- stream in fully coalesced; the few
//    tokens' u rows are broadcast reads.  The sum runs over k in ascending order on the vector
//    ALUs.
//
// A call may cover up to 4 target slots that read the same x (the query, key and value
// projections of a layer).
//
// HBM traffic: x once per slot, y read and written once, the factors once per adapter and launch (L2
// serves tiles that share one), u is a few KB per tile.
#include "lora_device.h"

#include <algorithm>

namespace tidal {

// Entry that owns work unit `unit`: the number of later entries whose first unit is <= unit.
// Uniform per wave; the reads do not depend on each other.
__device__ __forceinline__ int find_entry(const ApplyLongBatch& batch, int unit) {
    int si = 0;
#pragma unroll
    for (int k = 1; k < kMaxApplyLong; ++k) si += batch.first[k] <= unit ? 1 : 0;
    return si;
}

// One (short segment, slot) pair with its tables resolved.
struct ApplyEntry {
    const uint16_t* Ar;
    const uint16_t* Bp;
    uint16_t* y;
    int t0, rows;
    float s;
    int r, rp, out;
    uint32_t u_tok;
};
__device__ __forceinline__ ApplyEntry resolve(const ApplyShortBatch& batch, int si, int slot) {
    const ApplyShortSeg g = batch.seg[si];
    const ApplyFactor f = batch.fac[g.fac + slot];
    const ApplySlot sl = batch.slot[slot];
    ApplyEntry e;
    e.Ar = (const uint16_t*)(batch.adapter_base + (size_t)f.ar * kLoraUnit);
    e.Bp = (const uint16_t*)(batch.adapter_base + (size_t)f.bp * kLoraUnit);
    e.y = sl.y;
    e.t0 = g.t0;
    e.rows = g.rows;
    e.s = f.s;
    e.r = f.r;
    e.rp = f.rp;
    e.out = sl.out;
    e.u_tok = sl.u_tok;
    return e;
}

// ---------------------------------------------------------------------------------------
// shrink
// ---------------------------------------------------------------------------------------
constexpr int kShrinkWaves = 4;
constexpr int kStagePitch = 72;                                   // bf16 per staged row: 64 + 8 of padding
constexpr int kStageRows = 32 + 64;                               // x rows, then A rows
constexpr int kStageBytes = kStageRows * kStagePitch * 2;         // 13,824 per wave
constexpr int kPartBytes = kShrinkWaves * 2 * 32 * 32 * 4;        // 32,768
constexpr int kShrinkLds = kShrinkWaves * kStageBytes > kPartBytes ? kShrinkWaves * kStageBytes : kPartBytes;

__device__ __forceinline__ u32x4 zero4() {
    const u32x4 z = {0u, 0u, 0u, 0u};
    return z;
}

// Full-line fetch of one 64-column group: lane l takes 16 bytes at row (l / 8 + 8 i), piece l % 8.
// XI = number of x row blocks (rows / 8 rounded up), AI likewise for the A rows.
template <int XI, int AI>
__device__ __forceinline__ void fetch_group(const uint16_t* __restrict__ x, const uint16_t* __restrict__ Ar, int in,
                                            int rows, int r, int j0, int lane, u32x4 (&xr)[4], u32x4 (&ar)[8]) {
    const int sub = lane >> 3, piece = lane & 7;
    const int j = j0 + 8 * piece;
    const bool col_ok = j + 8 <= in;                              // in is a multiple of 8
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        const int row = sub + 8 * i;
        xr[i] = (col_ok && row < rows) ? *as_global((const u32x4*)(x + (int64_t)row * in + j)) : zero4();
    }
#pragma unroll
    for (int i = 0; i < AI; ++i) {
        const int row = sub + 8 * i;
        ar[i] = (col_ok && row < r) ? *as_global((const u32x4*)(Ar + (int64_t)row * in + j)) : zero4();
    }
}

// One group: park the fetched registers in the wave's stage, multiply from there.
template <int XI, int AI>
__device__ __forceinline__ void shrink_group(uint16_t* xs, uint16_t* as, int lane, const u32x4 (&xr)[4],
                                             const u32x4 (&ar)[8], f32x16& c0, f32x16& c1) {
    constexpr bool TWO = AI > 4;
    const int sub = lane >> 3, piece = lane & 7;
    const int n = lane & 31, kg = lane >> 5;
#pragma unroll
    for (int i = 0; i < XI; ++i) *(u32x4*)(xs + (sub + 8 * i) * kStagePitch + 8 * piece) = xr[i];
#pragma unroll
    for (int i = 0; i < AI; ++i) *(u32x4*)(as + (sub + 8 * i) * kStagePitch + 8 * piece) = ar[i];
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const bf16x8 xo = *(const bf16x8*)(xs + n * kStagePitch + 16 * q + 8 * kg);
        const bf16x8 a0 = *(const bf16x8*)(as + n * kStagePitch + 16 * q + 8 * kg);
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xo, a0, c0, 0, 0, 0);
        if constexpr (TWO) {
            const bf16x8 a1 = *(const bf16x8*)(as + (32 + n) * kStagePitch + 16 * q + 8 * kg);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xo, a1, c1, 0, 0, 0);
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// A single workgroup sees one load latency per group unless several groups are in flight: three
// groups' worth of registers rotate (two at 64 ranks, where a group is 12 vectors per lane).
template <int XI, int AI, int W = kShrinkWaves>
__device__ __forceinline__ void shrink_walk(const uint16_t* __restrict__ x, const uint16_t* __restrict__ Ar, int in,
                                            int rows, int r, int lane, int wave, uint16_t* stage, f32x16& c0,
                                            f32x16& c1) {
    // groups of registers in flight: the fewer vectors a group is, the more of them fit (measured on the
    // 8 x 512-token batch: 6 deep for groups of up to 4 vectors, 25.6 -> 24.7 us; 4 deep for 5-6 vectors lost 2 %)
    constexpr int D = (XI + AI) <= 4 ? 6 : ((XI + AI) <= 8 ? 3 : 2);
    const int groups = (in + 63) >> 6;
    const int sub = lane >> 3, piece = lane & 7;
    uint16_t* xs = stage;
    uint16_t* as = stage + 32 * kStagePitch;
    // rows that are never fetched must read as zeros (ranks r..rp-1) or at least as numbers
    for (int row = sub; row < kStageRows; row += 8) *(u32x4*)(stage + row * kStagePitch + 8 * piece) = zero4();

    u32x4 xb[D][4], ab[D][8];
    int g = wave;
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (g + d * W < groups) fetch_group<XI, AI>(x, Ar, in, rows, r, (g + d * W) * 64, lane, xb[d], ab[d]);
    for (; g < groups; g += D * W) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            if (g + d * W < groups) {
                shrink_group<XI, AI>(xs, as, lane, xb[d], ab[d], c0, c1);
                if (g + (D + d) * W < groups)
                    fetch_group<XI, AI>(x, Ar, in, rows, r, (g + (D + d) * W) * 64, lane, xb[d], ab[d]);
            }
        }
    }
}

__global__ __launch_bounds__(64 * kShrinkWaves) void apply_shrink_kernel(const ApplyLongBatch batch, int in) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[kShrinkLds];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int si = find_entry(batch, blockIdx.x);
    const ApplyLongEntry sg = batch.e[si];
    const int tile0 = sg.t0 + 32 * ((int)blockIdx.x - batch.first[si]);   // first token of this tile
    const int rows = sg.t1 - tile0 < 32 ? sg.t1 - tile0 : 32;
    const uint16_t* x = batch.x + (int64_t)tile0 * in;
    uint16_t* stage = (uint16_t*)(lds + wave * kStageBytes);

    f32x16 c0 = {0}, c1 = {0};
    const int xi = (rows + 7) >> 3;
    // instantiations by the number of 8-row blocks to fetch: x 1 or 4, A 2, 4 or 8
    if (sg.rp == 16) {
        if (xi == 1) shrink_walk<1, 2>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else shrink_walk<4, 2>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
    } else if (sg.rp == 32) {
        if (xi == 1) shrink_walk<1, 4>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else shrink_walk<4, 4>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
    } else {
        if (xi == 1) shrink_walk<1, 8>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else shrink_walk<4, 8>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
    }

    // C layout: lane holds rank column n of token rows 8*(v/4) + 4*kg + v%4
    const int n = lane & 31, kg = lane >> 5;
    const bool two = sg.rp > 32;
    __syncthreads();                                              // the stages become the partial sums
    float* part = (float*)lds;                                    // [wave][rank tile][token][rank]
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = 8 * (v >> 2) + 4 * kg + (v & 3);
        part[((wave * 2 + 0) * 32 + row) * 32 + n] = c0[v];
        if (two) part[((wave * 2 + 1) * 32 + row) * 32 + n] = c1[v];
    }
    __syncthreads();
    uint32_t* u = (uint32_t*)(batch.u + ((int64_t)sg.u_tok + sg.t0) * kApplyRankStride + (int64_t)(tile0 - sg.t0) * sg.rp);
    const int pairs_per_row = sg.rp >> 1;
    const int pairs = rows * pairs_per_row;
    for (int e = threadIdx.x; e < pairs; e += 64 * kShrinkWaves) {
        const int row = e / pairs_per_row;
        const int k = 2 * (e - row * pairs_per_row);
        float lo = 0.0f, hi = 0.0f;
#pragma unroll
        for (int w = 0; w < kShrinkWaves; ++w) {                  // fixed order: reproducible
            lo += part[((w * 2 + (k >> 5)) * 32 + row) * 32 + (k & 31)];
            hi += part[((w * 2 + (k >> 5)) * 32 + row) * 32 + (k & 31) + 1];
        }
        const f32x2 r2 = {lo, hi};
        as_global(u)[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(r2, bf16x2));
    }
}

hipError_t launch_apply_shrink(const ApplyLongBatch& b, int n_tiles, int in, hipStream_t stream) {
    if (n_tiles <= 0) return hipSuccess;
    if (b.n <= 0 || b.n > kMaxApplyLong || in <= 0 || in % 8) return hipErrorInvalidValue;
    hipLaunchKernelGGL(apply_shrink_kernel, dim3((unsigned)n_tiles), dim3(64 * kShrinkWaves), 0, stream, b, in);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// prompts in one launch: shrink and expand of a token tile in the same workgroup
// ---------------------------------------------------------------------------------------
// A workgroup of 8 waves owns one tile of 32 (or, NV = 8, 16) token rows of one entry.  The waves
// split the input width for u = bf16(A x) exactly as in apply_shrink_kernel, the partial tiles meet
// in LDS and are added in wave order, and u stays in LDS: each wave then takes every eighth strip
// of 256 outputs and updates its piece of y with the register tiling of the in-place merge (y in
// the place of W, u as the per-row factor, B's rows as the strip).  No intermediate reaches
// memory and the two steps need no second launch -- for a prompt batch of a few thousand tokens a
// launch's ramp-up and tail are as long as its data movement.  Small batches take 16-row tiles so
// that every compute unit gets a workgroup; the upper half of the matrix-core tile then idles.
// (Workgroups of 4 waves, two per compute unit so that one's shrink overlaps the other's expand,
// each wave walking two of the eight parts of the input width, were measured on a 16,384-token
// prompt: 106 us against 85.)
constexpr int kFusedWaves = 8;
constexpr int kFusedPartBytes = kFusedWaves * 2 * 32 * 32 * 4;    // 65,536
constexpr int kFusedLds = kFusedWaves * kStageBytes;              // 110,592: the stages; later partial sums + u
static_assert(kFusedPartBytes + 32 * 64 * 2 <= kFusedLds, "partial sums and u must fit where the stages were");

// The lane's part of a tile of y for one strip of 256 outputs: rows 8*(v/4) + 4*h + v%4 (v < NV), 8
// adjacent outputs each.  Interior pieces use one vector access per row, ragged ones go by element.
template <int NV>
__device__ __forceinline__ void y_fetch(const uint16_t* __restrict__ y, int out, int rows, int strip, int lane,
                                        uint32_t (&w)[NV][4]) {
    typedef typename RowVec<8>::type vec_t;
    const int n = lane & 31, h = lane >> 5;
    const int j0 = strip << 8, jl = j0 + 8 * n;
    if (j0 + 256 <= out && rows == 2 * NV) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int row = 8 * (v >> 2) + 4 * h + (v & 3);
            unpack_words<8>(load_w((const vec_t*)(y + (int64_t)row * out + jl)), w[v]);
        }
    } else {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int row = 8 * (v >> 2) + 4 * h + (v & 3);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                uint32_t lo = 0, hi = 0;
                if (row < rows && jl + 2 * p < out) lo = as_global(y)[(int64_t)row * out + jl + 2 * p];
                if (row < rows && jl + 2 * p + 1 < out) hi = as_global(y)[(int64_t)row * out + jl + 2 * p + 1];
                w[v][p] = lo | (hi << 16);
            }
        }
    }
}

template <int NV>
__device__ __forceinline__ void y_store(uint16_t* __restrict__ y, int out, int rows, int strip, int lane,
                                        const uint32_t (&w)[NV][4]) {
    typedef typename RowVec<8>::type vec_t;
    const int n = lane & 31, h = lane >> 5;
    const int j0 = strip << 8, jl = j0 + 8 * n;
    if (j0 + 256 <= out && rows == 2 * NV) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int row = 8 * (v >> 2) + 4 * h + (v & 3);
            store_w((vec_t*)(y + (int64_t)row * out + jl), pack_words<8>(w[v]));
        }
    } else {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int row = 8 * (v >> 2) + 4 * h + (v & 3);
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                if (row < rows && jl + 2 * p < out) as_global(y)[(int64_t)row * out + jl + 2 * p] = (uint16_t)(w[v][p] & 0xFFFFu);
                if (row < rows && jl + 2 * p + 1 < out) as_global(y)[(int64_t)row * out + jl + 2 * p + 1] = (uint16_t)(w[v][p] >> 16);
            }
        }
    }
}

// w += s * (u B^T) for one strip: u (token rows) is the matrix-core A operand, B's rows for the
// lane's 8 outputs the B operand, TB of them at a time (all 8 would not fit the registers at 64 ranks).
template <int KS, int NV>
__device__ __forceinline__ void strip_update(const ApplyLongEntry& sg, const bf16x8 (&aop)[KS], int strip, int lane,
                                             uint32_t (&w)[NV][4]) {
    constexpr int NT = 8;
    constexpr int TB = KS == 4 ? 4 : NT;
    const int n = lane & 31, h = lane >> 5;
    const int out = sg.out, jl = (strip << 8) + NT * n;
    const TIDAL_GLOBAL bf16x8* g = as_global((const bf16x8*)sg.Bp);
#pragma unroll
    for (int tb = 0; tb < NT; tb += TB) {
        bf16x8 bop[TB][KS];
#pragma unroll
        for (int T = 0; T < TB; ++T) {
            int j = jl + tb + T;
            j = j < out ? j : out - 1;                            // ragged strip: clamp, masked at the store
            const int64_t base = bp_group(j, 0, h, KS);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) bop[T][ks] = g[base + 64 * ks];
        }
#pragma unroll
        for (int q = 0; q < TB / 2; ++q) {
            f32x16 c0 = {0}, c1 = {0};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], bop[2 * q][ks], c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks], bop[2 * q + 1][ks], c1, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < NV; ++v) w[v][tb / 2 + q] = rmw2(w[v][tb / 2 + q], c0[v], c1[v], sg.s);
        }
    }
}

// The wave's strips (every eighth), two at a time: the second one's y is on its way while the first
// is updated, where the registers allow.  EARLY: w0 arrives holding the wave's first strip.
template <int KS, int NV, bool EARLY>
__device__ __forceinline__ void fused_expand(const ApplyLongEntry& sg, const uint16_t* u_lds, uint16_t* y, int rows,
                                             int wave, int lane, uint32_t (&w0)[NV][4]) {
    constexpr bool AHEAD = NV == 8 && KS <= 2;
    const int out = sg.out;
    const int strips = (out + 255) >> 8;
    const int n = lane & 31, h = lane >> 5;
    bf16x8 aop[KS];                                               // token row n, ranks 16 ks + 8 h + 0..7
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) aop[ks] = *(const bf16x8*)(u_lds + n * (16 * KS) + 16 * ks + 8 * h);
    for (int strip = wave; strip < strips; strip += 2 * kFusedWaves) {
        const int next = strip + kFusedWaves;
        uint32_t w1[NV][4];
        if (!EARLY || strip != wave) y_fetch<NV>(y, out, rows, strip, lane, w0);
        if constexpr (AHEAD) {
            if (next < strips) y_fetch<NV>(y, out, rows, next, lane, w1);
        }
        strip_update<KS, NV>(sg, aop, strip, lane, w0);
        y_store<NV>(y, out, rows, strip, lane, w0);
        if (next < strips) {
            if constexpr (!AHEAD) y_fetch<NV>(y, out, rows, next, lane, w1);
            strip_update<KS, NV>(sg, aop, next, lane, w1);
            y_store<NV>(y, out, rows, next, lane, w1);
        }
    }
}

// NV = rows of a tile that a lane owns: 16 (32-token tiles) or 8 (16-token tiles)
template <int NV>
__global__ __launch_bounds__(64 * kFusedWaves) void apply_fused_kernel(const ApplyLongBatch batch, int in) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[kFusedLds];
    constexpr int TR = 2 * NV;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int si = find_entry(batch, blockIdx.x);
    const ApplyLongEntry sg = batch.e[si];
    const int tile0 = sg.t0 + TR * ((int)blockIdx.x - batch.first[si]);   // first token of this tile
    const int rows = sg.t1 - tile0 < TR ? sg.t1 - tile0 : TR;
    const uint16_t* x = batch.x + (int64_t)tile0 * in;
    uint16_t* stage = (uint16_t*)(lds + wave * kStageBytes);

    f32x16 c0 = {0}, c1 = {0};
    const int xi = (rows + 7) >> 3;
    // instantiations by the number of 8-row blocks to fetch: x 1, 2 or 4, A 2, 4 or 8
    if (sg.rp == 16) {
        if (xi == 1) shrink_walk<1, 2, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else if (xi == 2) shrink_walk<2, 2, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else shrink_walk<4, 2, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
    } else if (sg.rp == 32) {
        if (xi == 1) shrink_walk<1, 4, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else if (xi == 2) shrink_walk<2, 4, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else shrink_walk<4, 4, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
    } else {
        if (xi == 1) shrink_walk<1, 8, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else if (xi == 2) shrink_walk<2, 8, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
        else shrink_walk<4, 8, kFusedWaves>(x, sg.Ar, in, rows, sg.r, lane, wave, stage, c0, c1);
    }

    // y does not depend on u: the wave's first strip sets out now and arrives during the reduction
    uint16_t* y = sg.y + (int64_t)tile0 * sg.out;
    uint32_t w0[NV][4];
    constexpr bool EARLY = NV == 8;                               // 32-token tiles: the registers do not allow it
    if constexpr (EARLY) {
        if (wave < ((sg.out + 255) >> 8)) y_fetch<NV>(y, sg.out, rows, wave, lane, w0);
    }

    // C layout: lane holds rank column n of token rows 8*(v/4) + 4*kg + v%4
    const int n = lane & 31, kg = lane >> 5;
    const bool two = sg.rp > 32;
    __syncthreads();                                              // the stages become the partial sums
    float* part = (float*)lds;                                    // [wave][rank tile][token][rank]
#pragma unroll
    for (int v = 0; v < NV; ++v) {                                // the tile's rows: 8*(v/4) + 4*kg + v%4 < 2*NV
        const int row = 8 * (v >> 2) + 4 * kg + (v & 3);
        part[((wave * 2 + 0) * 32 + row) * 32 + n] = c0[v];
        if (two) part[((wave * 2 + 1) * 32 + row) * 32 + n] = c1[v];
    }
    __syncthreads();
    uint16_t* u_lds = (uint16_t*)(lds + kFusedPartBytes);         // 32 token rows x rp bf16; rows past the tile's are zeros
    const int pairs_per_row = sg.rp >> 1;
    for (int e = threadIdx.x; e < 32 * pairs_per_row; e += 64 * kFusedWaves) {
        const int row = e / pairs_per_row;
        const int k = 2 * (e - row * pairs_per_row);
        float lo = 0.0f, hi = 0.0f;
        if (row < TR) {
#pragma unroll
            for (int w = 0; w < kFusedWaves; ++w) {               // fixed order: reproducible
                lo += part[((w * 2 + (k >> 5)) * 32 + row) * 32 + (k & 31)];
                hi += part[((w * 2 + (k >> 5)) * 32 + row) * 32 + (k & 31) + 1];
            }
        }
        const f32x2 r2 = {lo, hi};
        ((uint32_t*)u_lds)[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(r2, bf16x2));
    }
    __syncthreads();
    if (sg.rp == 16) fused_expand<1, NV, EARLY>(sg, u_lds, y, rows, wave, lane, w0);
    else if (sg.rp == 32) fused_expand<2, NV, EARLY>(sg, u_lds, y, rows, wave, lane, w0);
    else fused_expand<4, NV, EARLY>(sg, u_lds, y, rows, wave, lane, w0);
}

// tile_rows: 32 or 16 (token rows per workgroup; first[] of the batch counts tiles of that height)
hipError_t launch_apply_fused(const ApplyLongBatch& b, int n_tiles, int tile_rows, int in, hipStream_t stream) {
    if (n_tiles <= 0) return hipSuccess;
    if (b.n <= 0 || b.n > kMaxApplyLong || in <= 0 || in % 8) return hipErrorInvalidValue;
    for (int k = 0; k < b.n; ++k)
        if (b.e[k].out <= 0 || b.e[k].out % 8 || (b.e[k].rp != 16 && b.e[k].rp != 32 && b.e[k].rp != 64))
            return hipErrorInvalidValue;
    if (tile_rows == 32) hipLaunchKernelGGL(apply_fused_kernel<16>, dim3((unsigned)n_tiles), dim3(64 * kFusedWaves), 0, stream, b, in);
    else if (tile_rows == 16) hipLaunchKernelGGL(apply_fused_kernel<8>, dim3((unsigned)n_tiles), dim3(64 * kFusedWaves), 0, stream, b, in);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

__device__ __forceinline__ void unpack8(const u32x4 v, float (&f)[8]) {
    const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        f[2 * e] = __uint_as_float(wds[e] << 16);
        f[2 * e + 1] = __uint_as_float(wds[e] & 0xFFFF0000u);
    }
}

// ---------------------------------------------------------------------------------------
// shrink, few tokens per segment: one wave per rank row
// ---------------------------------------------------------------------------------------
// A wave owns rank row k of one segment: its lanes stride along the input width in 16-byte
// pieces (1 KB per wave-wide load, fully coalesced), multiply with the segment's x rows and
// reduce across lanes once per token at the end.  Four rank rows per workgroup, so a decode
// batch of 64 requests at rank 16 is 256 workgroups whose loads are all independent.
// (Four rank rows per wave, with x fetched once for the four, moves a quarter of the x through the
// L2 and was measured slower all the same -- 31 against 18 us per call for 64 requests, 37 against
// 31 for 256: these launches live on the number of independent loads in flight, not on bytes.)
__global__ __launch_bounds__(256) void apply_shrink_short_kernel(const ApplyShortBatch batch, int in) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int e = blockIdx.x >> 4;                                // 16 workgroups per (segment, slot): 64 rank rows
    const int k = ((blockIdx.x & 15) << 2) + wave;
    const int si = e / batch.n_slots;
    const ApplyEntry sg = resolve(batch, si, e - si * batch.n_slots);
    if (sg.r == 0 || k >= sg.rp) return;
    const int rows = sg.rows;                                     // 1 .. kApplyShortRows
    float acc[kApplyShortRows];
#pragma unroll
    for (int t = 0; t < kApplyShortRows; ++t) acc[t] = 0.0f;
    if (k < sg.r) {
        const uint16_t* arow = sg.Ar + (int64_t)k * in;
        const uint16_t* x = batch.x + (int64_t)sg.t0 * in;
#pragma unroll 8
        for (int j = 8 * lane; j < in; j += 512) {               // in is a multiple of 8
            float a8[8];
            const u32x4 av = *as_global((const u32x4*)(arow + j));
            unpack8(av, a8);
#pragma unroll
            for (int t = 0; t < kApplyShortRows; ++t) {
                if (t < rows) {
                    float x8[8];
                    const u32x4 xv = *as_global((const u32x4*)(x + (int64_t)t * in + j));
                    unpack8(xv, x8);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[t] = __builtin_fmaf(a8[e], x8[e], acc[t]);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < kApplyShortRows; ++t)
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) acc[t] += __shfl_xor(acc[t], off, 64);
    }
    if (lane < rows) {                                            // lane t stores token t's value (zero for padded ranks)
        float v = acc[0];
#pragma unroll
        for (int t = 1; t < kApplyShortRows; ++t) v = lane == t ? acc[t] : v;
        const f32x2 r2 = {v, 0.0f};
        as_global(batch.u)[((int64_t)sg.u_tok + sg.t0) * kApplyRankStride + lane * sg.rp + k] =
            (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(r2, bf16x2)) & 0xFFFFu);
    }
}

hipError_t launch_apply_shrink_short(const ApplyShortBatch& b, int in, hipStream_t stream) {
    if (b.n_segs <= 0) return hipSuccess;
    if (b.n_segs > kMaxApplyShort || b.n_slots <= 0 || b.n_slots > kMaxApplySlots || in <= 0 || in % 8)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(apply_shrink_short_kernel, dim3((unsigned)(b.n_segs * b.n_slots * 16)), dim3(256), 0, stream, b, in);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// expand, matrix cores
// ---------------------------------------------------------------------------------------
template <int KS>
__device__ __forceinline__ void expand_walk(const ApplyLongBatch& batch, const ApplyLongEntry& sg, int t_begin,
                                            int chunk_rows, int j0, int lane) {
    const int out = sg.out;
    constexpr int NT = 8;
    bf16x8 bop[NT][KS];
    {   // rows of B for the lane's 8 outputs, gathered from the packed (operand-order) B
        const int n_ = lane & 31, kg = lane >> 5;
        const TIDAL_GLOBAL bf16x8* g = as_global((const bf16x8*)sg.Bp);
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            int j = j0 + NT * n_ + T;
            j = j < out ? j : out - 1;                           // ragged strip: clamp, masked at the store
            const int64_t base = bp_group(j, 0, kg, KS);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) bop[T][ks] = g[base + 64 * ks];
        }
    }
    const int n = lane & 31, h = lane >> 5;
    const int jl = j0 + NT * n;
    const bool strip_full = j0 + 32 * NT <= out;
    const int t_end = sg.t1 < t_begin + chunk_rows ? sg.t1 : t_begin + chunk_rows;
    for (int t = t_begin; t < t_end; t += 32) {
        const int rows = t_end - t < 32 ? t_end - t : 32;
        const uint16_t* u = batch.u + ((int64_t)sg.u_tok + sg.t0) * kApplyRankStride + (int64_t)(t - sg.t0) * sg.rp;
        uint16_t* y = sg.y + (int64_t)t * out;
        const bool full = strip_full && rows == 32;
        uint32_t w[16][NT / 2];
        load_block<NT>(y, rows, out, 0, jl, h, full, w);
        f32x16 acc[NT];
        bf16x8 aop[KS];
        load_rows<KS>(u, rows, 0, lane, aop);
        delta_tile<NT, KS>(aop, bop, acc);
        apply_tile<NT>(w, acc, sg.s);
        store_block<NT>(y, rows, out, 0, jl, h, full, w);
    }
}

// KS = padded rank / 16 of every entry of the launch (one kernel with all three bodies would need
// the registers of the largest and run the small ranks at half their occupancy).
template <int KS>
__global__ __launch_bounds__(256) void apply_expand_kernel(const ApplyLongBatch batch, int n_chunks, int chunk_rows,
                                                           int strips) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t item = (int64_t)blockIdx.x * 4 + wave;
    if (item >= (int64_t)n_chunks * strips) return;
    // the four waves of a workgroup take neighbouring strips of one chunk: adjacent pieces of the same y rows
    const int chunk = (int)(item / strips);
    const int strip = (int)(item - (int64_t)chunk * strips);
    const int si = find_entry(batch, chunk);
    const ApplyLongEntry sg = batch.e[si];
    if (strip * 256 >= sg.out) return;                            // strips are counted for the widest slot
    const int t_begin = sg.t0 + chunk_rows * (chunk - batch.first[si]);
    expand_walk<KS>(batch, sg, t_begin, chunk_rows, strip * 256, lane);
}

// rp: the padded rank of every entry of the launch
hipError_t launch_apply_expand(const ApplyLongBatch& b, int n_chunks, int chunk_tiles, int max_out, int rp,
                               hipStream_t stream) {
    if (n_chunks <= 0) return hipSuccess;
    if (b.n <= 0 || b.n > kMaxApplyLong || max_out <= 0 || chunk_tiles < 1) return hipErrorInvalidValue;
    for (int k = 0; k < b.n; ++k)
        if (b.e[k].out <= 0 || b.e[k].out % 8 || b.e[k].out > max_out || b.e[k].rp != rp) return hipErrorInvalidValue;
    const int strips = (max_out + 255) / 256;
    const int64_t items = (int64_t)n_chunks * strips;
    if ((items + 3) / 4 > 0x7FFFFFF0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((items + 3) / 4));
    const int chunk_rows = 32 * chunk_tiles;
    switch (rp) {
        case 16: hipLaunchKernelGGL(apply_expand_kernel<1>, grid, dim3(256), 0, stream, b, n_chunks, chunk_rows, strips); break;
        case 32: hipLaunchKernelGGL(apply_expand_kernel<2>, grid, dim3(256), 0, stream, b, n_chunks, chunk_rows, strips); break;
        case 64: hipLaunchKernelGGL(apply_expand_kernel<4>, grid, dim3(256), 0, stream, b, n_chunks, chunk_rows, strips); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// expand, few tokens per segment: one lane per output
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void apply_expand_short_kernel(const ApplyShortBatch batch, int blocks_per_seg) {
    const int e = blockIdx.x / blocks_per_seg;                    // (segment, slot), slots fastest
    const int i = (blockIdx.x - e * blocks_per_seg) * 256 + threadIdx.x;
    const int si = e / batch.n_slots;
    const ApplyEntry sg = resolve(batch, si, e - si * batch.n_slots);
    const int out = sg.out;
    if (sg.r == 0 || i >= out) return;
    const int rows = sg.rows;                                     // 1 .. kApplyShortRows
    const uint16_t* u = batch.u + ((int64_t)sg.u_tok + sg.t0) * kApplyRankStride;
    const TIDAL_GLOBAL u32x4* bgroups = as_global((const u32x4*)sg.Bp);      // packed B: 16-byte groups of 8 ranks
    const int KS = sg.rp >> 4;
    float acc[kApplyShortRows], yv[kApplyShortRows];
#pragma unroll
    for (int t = 0; t < kApplyShortRows; ++t) {
        acc[t] = 0.0f;
        yv[t] = 0.0f;
        if (t < rows) yv[t] = __uint_as_float((uint32_t)as_global(sg.y)[(int64_t)(sg.t0 + t) * out + i] << 16);
    }
    for (int k0 = 0; k0 < sg.rp; k0 += 8) {
        float b8[8];
        const u32x4 bv = bgroups[bp_group(i, k0 >> 4, (k0 >> 3) & 1, KS)];
        unpack8(bv, b8);
#pragma unroll
        for (int t = 0; t < kApplyShortRows; ++t) {
            if (t < rows) {
                float u8[8];
                const u32x4 uv = *as_global((const u32x4*)(u + t * sg.rp + k0));
                unpack8(uv, u8);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[t] = __builtin_fmaf(b8[e], u8[e], acc[t]);
            }
        }
    }
#pragma unroll
    for (int t = 0; t < kApplyShortRows; ++t) {
        if (t < rows) {
            const f32x2 r2 = {__builtin_fmaf(sg.s, acc[t], yv[t]), 0.0f};
            as_global(sg.y)[(int64_t)(sg.t0 + t) * out + i] =
                (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(r2, bf16x2)) & 0xFFFFu);
        }
    }
}

hipError_t launch_apply_expand_short(const ApplyShortBatch& b, int max_out, hipStream_t stream) {
    if (b.n_segs <= 0) return hipSuccess;
    if (b.n_segs > kMaxApplyShort || b.n_slots <= 0 || b.n_slots > kMaxApplySlots || max_out <= 0) return hipErrorInvalidValue;
    const int blocks_per_seg = (max_out + 255) / 256;
    hipLaunchKernelGGL(apply_expand_short_kernel, dim3((unsigned)(b.n_segs * b.n_slots * blocks_per_seg)), dim3(256), 0,
                       stream, b, blocks_per_seg);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// ordered accumulation (TIDAL_FLAG_ORDERED_ACCUM): both sums as one fused multiply-add chain in
// ascending index order, the order a sequential definition takes -- reproducible bit for bit,
// and slow: one lane per u[t][k] walks the whole input width.  Entries as for the prompts.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void apply_ordered_shrink_kernel(const ApplyLongBatch batch, int in) {
    const ApplyLongEntry sg = batch.e[blockIdx.y];
    const int rows = sg.t1 - sg.t0;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)rows * sg.rp) return;
    const int t = (int)(idx / sg.rp), k = (int)(idx - (int64_t)t * sg.rp);
    float acc = 0.0f;
    if (k < sg.r) {
        const TIDAL_GLOBAL uint16_t* a = as_global(sg.Ar + (int64_t)k * in);
        const TIDAL_GLOBAL uint16_t* x = as_global(batch.x + (int64_t)(sg.t0 + t) * in);
        for (int j = 0; j < in; ++j)
            acc = __builtin_fmaf(__uint_as_float((uint32_t)a[j] << 16), __uint_as_float((uint32_t)x[j] << 16), acc);
    }
    const f32x2 r2 = {acc, 0.0f};
    as_global(batch.u)[((int64_t)sg.u_tok + sg.t0) * kApplyRankStride + (int64_t)t * sg.rp + k] =
        (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(r2, bf16x2)) & 0xFFFFu);
}

__global__ __launch_bounds__(256) void apply_ordered_expand_kernel(const ApplyLongBatch batch) {
    const ApplyLongEntry sg = batch.e[blockIdx.y];
    const int rows = sg.t1 - sg.t0;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)rows * sg.out) return;
    const int t = (int)(idx / sg.out), i = (int)(idx - (int64_t)t * sg.out);
    const TIDAL_GLOBAL uint16_t* b = as_global(sg.Bp);
    const TIDAL_GLOBAL uint16_t* u = as_global(batch.u + ((int64_t)sg.u_tok + sg.t0) * kApplyRankStride + (int64_t)t * sg.rp);
    const int KS = sg.rp >> 4;
    float acc = 0.0f;
    for (int k = 0; k < sg.r; ++k) {
        const uint16_t bk = b[bp_group(i, k >> 4, (k >> 3) & 1, KS) * 8 + (k & 7)];
        acc = __builtin_fmaf(__uint_as_float((uint32_t)bk << 16), __uint_as_float((uint32_t)u[k] << 16), acc);
    }
    TIDAL_GLOBAL uint16_t* y = as_global(sg.y + (int64_t)(sg.t0 + t) * sg.out + i);
    const f32x2 r2 = {__builtin_fmaf(sg.s, acc, __uint_as_float((uint32_t)*y << 16)), 0.0f};
    *y = (uint16_t)(__builtin_bit_cast(uint32_t, __builtin_convertvector(r2, bf16x2)) & 0xFFFFu);
}

hipError_t launch_apply_ordered(const ApplyLongBatch& b, int in, bool shrink, hipStream_t stream) {
    if (b.n <= 0) return hipSuccess;
    if (b.n > kMaxApplyLong || in <= 0) return hipErrorInvalidValue;
    int64_t most = 0;
    for (int k = 0; k < b.n; ++k) {
        const int64_t rows = (int64_t)b.e[k].t1 - b.e[k].t0;
        most = std::max(most, rows * (shrink ? b.e[k].rp : b.e[k].out));
    }
    const int64_t blocks = (most + 255) / 256;
    if (blocks <= 0) return hipSuccess;
    if (blocks > 0x7FFFFFF0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks, (unsigned)b.n);
    if (shrink) hipLaunchKernelGGL(apply_ordered_shrink_kernel, grid, dim3(256), 0, stream, b, in);
    else hipLaunchKernelGGL(apply_ordered_expand_kernel, grid, dim3(256), 0, stream, b);
    return hipGetLastError();
}

}  // namespace tidal
