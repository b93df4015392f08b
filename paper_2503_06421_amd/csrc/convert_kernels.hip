// Narrowing of staged checkpoint data to bf16 template slots, and packing of LoRA
// factors into the layout the merge kernels read.  gfx950 only.
//
// The paper treats dtype changes and host-to-GPU copies as the operators that produce
// a weight (Sec. 4.1, weight-centric tracing); here the dtype change is one streaming
// kernel per staged chunk.  It is bound by HBM traffic (4 or 2 bytes in, 2 bytes out per
// element, no reuse), so every lane moves 16-byte vectors and the arithmetic is the
// hardware's IEEE conversions: round to nearest even, subnormals kept, infinities kept,
// NaN quieted with sign and upper payload kept.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tidal_internal.h"

namespace tidal {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// Two binary32 -> two bf16 in one word (low half = first).  v_cvt_pk_bf16_f32 rounds to
// nearest even, keeps subnormals and quiets NaN keeping sign and upper payload: the same
// function as (u + 0x7FFF + ((u >> 16) & 1)) >> 16 with NaN -> (u >> 16) | 0x40 on all 2^32
// inputs (checked exhaustively on gfx950).
__device__ __forceinline__ uint32_t narrow2_f32(uint32_t a, uint32_t b) {
    const f32x2 v = {__uint_as_float(a), __uint_as_float(b)};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Two binary16 (one word) -> two bf16.  binary16 -> binary32 is exact in hardware (subnormals
// included: the kernel runs with denormals enabled); a signalling NaN is quieted on the way,
// which the bf16 narrowing would do anyway, and the payload bits that survive are the same.
__device__ __forceinline__ uint32_t narrow2_f16(uint32_t two) {
    const f16x2 h = __builtin_bit_cast(f16x2, two);
    const f32x2 v = {(float)h.x, (float)h.y};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 8 elements per lane per step.
__device__ __forceinline__ u32x4 narrow8_f32(u32x4 a, u32x4 b) {
    u32x4 o;
    o.x = narrow2_f32(a.x, a.y);
    o.y = narrow2_f32(a.z, a.w);
    o.z = narrow2_f32(b.x, b.y);
    o.w = narrow2_f32(b.z, b.w);
    return o;
}

__device__ __forceinline__ u32x4 narrow8_f16(u32x4 a) {
    u32x4 o;
    o.x = narrow2_f16(a.x);
    o.y = narrow2_f16(a.y);
    o.z = narrow2_f16(a.z);
    o.w = narrow2_f16(a.w);
    return o;
}

__device__ __forceinline__ uint32_t pack2(uint32_t lo_bf16, uint32_t hi_bf16) {
    return lo_bf16 | (hi_bf16 << 16);
}

__device__ __forceinline__ uint16_t narrow1(const void* src, int dtype, int64_t i) {
    if (dtype == TIDAL_F32) return (uint16_t)narrow2_f32(((const uint32_t*)src)[i], 0u);
    if (dtype == TIDAL_F16) return (uint16_t)narrow2_f16(((const uint16_t*)src)[i]);
    return ((const uint16_t*)src)[i];
}

// One launch converts every segment of a staged chunk: blockIdx.y selects the segment,
// blockIdx.x strides over its 8-element vectors.  Segment sources are 16-byte aligned
// inside the staging buffer and destinations are 16-byte aligned inside their slot.
__global__ __launch_bounds__(256) void convert_segments_kernel(ConvertBatch batch) {
    const ConvertSegment seg = batch.seg[blockIdx.y];
    const int64_t nvec = seg.elems >> 3;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    u32x4* __restrict__ dst = (u32x4*)seg.dst;
    if (seg.dtype == TIDAL_F32) {
        const u32x4* __restrict__ src = (const u32x4*)seg.src;
        for (; v < nvec; v += stride) {
            u32x4 a = __builtin_nontemporal_load(src + 2 * v);
            u32x4 b = __builtin_nontemporal_load(src + 2 * v + 1);
            dst[v] = narrow8_f32(a, b);
        }
    } else if (seg.dtype == TIDAL_F16) {
        const u32x4* __restrict__ src = (const u32x4*)seg.src;
        for (; v < nvec; v += stride) {
            u32x4 a = __builtin_nontemporal_load(src + v);
            dst[v] = narrow8_f16(a);
        }
    } else {
        const u32x4* __restrict__ src = (const u32x4*)seg.src;
        for (; v < nvec; v += stride) dst[v] = __builtin_nontemporal_load(src + v);
    }
    // ragged tail (< 8 elements), one block only
    if (blockIdx.x == 0) {
        int64_t i = (nvec << 3) + threadIdx.x;
        if (i < seg.elems) ((uint16_t*)seg.dst)[i] = narrow1(seg.src, seg.dtype, i);
    }
}

hipError_t launch_convert(const ConvertBatch& batch, int nseg, hipStream_t stream) {
    if (nseg <= 0) return hipSuccess;
    int64_t max_elems = 0;
    for (int i = 0; i < nseg; ++i) max_elems = batch.seg[i].elems > max_elems ? batch.seg[i].elems : max_elems;
    // One 16-byte vector per lane and as many short-lived workgroups as that takes: on this chip
    // a streaming kernel is fastest when waves do one load, one store and retire (the same
    // pattern loses 15-30 % of bandwidth as a grid-stride loop: 4.5 instead of 6.5 TB/s for
    // fp16 at 32 vectors per lane).
    int64_t blocks = (max_elems / 8 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > (1 << 22)) blocks = 1 << 22;
    dim3 grid((unsigned)blocks, (unsigned)nseg, 1);
    hipLaunchKernelGGL(convert_segments_kernel, grid, dim3(256), 0, stream, batch);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Small host->device copies by a kernel.  A copy-engine transfer followed by a kernel on the
// same stream costs a hand-over of tens of microseconds; for the few hundred KB of a small
// adapter that is more than the transfer itself.  Pinned host memory is mapped into the GPU's
// address space, so a kernel can fetch it over the link directly: 16 bytes per lane, one vector
// per lane.  Measured on this machine, copy + following kernel: 256 KiB 9.8 us against 22.4 us
// through the copy engine, 1 MiB 29 against 36 us; from 4 MiB on the copy engine is faster.
// ---------------------------------------------------------------------------
// One launch moves every run of a batch: blockIdx.y selects the run.
__global__ __launch_bounds__(256) void copy_from_host_kernel(const CopyBatch batch) {
    const CopyRun run = batch.run[blockIdx.y];
    const int64_t nvec = (int64_t)(run.bytes >> 4);
    const u32x4* __restrict__ src = (const u32x4*)run.src;
    u32x4* __restrict__ dst = (u32x4*)run.dst;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < nvec) dst[i] = __builtin_nontemporal_load(src + i);
    if (blockIdx.x == 0 && threadIdx.x < (run.bytes & 15))   // last bytes of a length that is no multiple of 16
        ((uint8_t*)(dst + nvec))[threadIdx.x] = ((const uint8_t*)(src + nvec))[threadIdx.x];
}

hipError_t launch_copy_from_host(const CopyBatch& batch, int nrun, hipStream_t stream) {
    if (nrun <= 0) return hipSuccess;
    if (nrun > kMaxCopyRuns) return hipErrorInvalidValue;
    uint64_t most = 0;
    for (int i = 0; i < nrun; ++i) {
        if ((uintptr_t)batch.run[i].src % 16 || (uintptr_t)batch.run[i].dst % 16) return hipErrorInvalidValue;
        most = batch.run[i].bytes > most ? batch.run[i].bytes : most;
    }
    const uint64_t blocks = most >= 16 ? ((most >> 4) + 255) / 256 : 1;
    if (blocks > 0x7FFFFFF0ull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(copy_from_host_kernel, dim3((unsigned)blocks, (unsigned)nrun, 1), dim3(256), 0, stream, batch);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Packing of LoRA factors.  Host layout: A is r x in, B is out x r, row-major, any of the
// three dtypes.  Device layout read by the merge kernels, rp = r rounded up to 16:
//   At : A transposed, ranks zero padded to rp: 16-byte groups of 8 consecutive ranks of one column
//   Bp : B, ranks zero padded to rp: 16-byte groups of 8 consecutive ranks of one row
// so that a lane fetches the 8 consecutive k it needs for one column (or row) with a single
// 16-byte load; the groups are stored in the order the matrix-core operands take them (256 columns
// or 32 rows per block, padding filled with zeros), so that a wave's load is one contiguous
// kilobyte.  One lane produces one such 16-byte group.
// ---------------------------------------------------------------------------
__host__ __device__ inline int64_t pack_lines_padded(const PackSegment& seg) {
    return seg.layout == kPackAt ? (seg.lines + 255) / 256 * 256 : (seg.layout == kPackBp ? (seg.lines + 31) / 32 * 32 : seg.lines);
}

// Eight consecutive source elements from element idx on (a 16-byte aligned address), narrowed to bf16.
__device__ __forceinline__ u32x4 load8_narrow(const void* src, int dtype, int64_t idx) {
    if (dtype == TIDAL_F32) {
        const u32x4* p = (const u32x4*)((const uint32_t*)src + idx);
        return narrow8_f32(p[0], p[1]);
    }
    const u32x4 v = *(const u32x4*)((const uint16_t*)src + idx);
    return dtype == TIDAL_F16 ? narrow8_f16(v) : v;
}

// Half `T & 1` of word `T >> 1` of two vectors of 8 bf16, side by side in one word: element T of
// `lo` in the low half, of `hi` in the high half.
template <int T>
__device__ __forceinline__ uint32_t pair_of(const u32x4& lo, const u32x4& hi) {
    const uint32_t a = lo[T >> 1], b = hi[T >> 1];
    return (T & 1) ? ((a >> 16) | (b & 0xFFFF0000u)) : ((a & 0xFFFFu) | (b << 16));
}

template <int T>
__device__ __forceinline__ u32x4 column_of(const u32x4 (&row)[8]) {
    u32x4 o;
    o.x = pair_of<T>(row[0], row[1]);
    o.y = pair_of<T>(row[2], row[3]);
    o.z = pair_of<T>(row[4], row[5]);
    o.w = pair_of<T>(row[6], row[7]);
    return o;
}

__global__ __launch_bounds__(256) void pack_adapter_kernel(PackBatch batch) {
    const PackSegment seg = batch.seg[blockIdx.y];
    const int groups_per_line = seg.rp >> 3;                 // 16-byte groups per packed line
    const int KS = seg.rp >> 4;
    const int64_t lines_pad = pack_lines_padded(seg);
    const int64_t ngroups = lines_pad * groups_per_line;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t first = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool aligned = (uintptr_t)seg.src % 16 == 0;
    u32x4* __restrict__ dst = (u32x4*)seg.dst;
    const u32x4 zero = {0u, 0u, 0u, 0u};
    if (seg.layout == kPackAt && aligned && seg.lines % 8 == 0) {
        // A lane takes 8 ranks x 8 columns: eight 16-byte reads along the rows of A (neighbouring lanes
        // read neighbouring pieces: whole cache lines), an 8 x 8 transpose in registers, eight 16-byte
        // groups out, each next to the one the neighbouring lane writes.
        const int64_t nblk = lines_pad >> 3;
        for (int64_t unit = first; unit < nblk * groups_per_line; unit += stride) {
            const int64_t c = unit % nblk;                    // block of 8 columns
            const int kg = (int)(unit / nblk);
            u32x4 row[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int k = kg * 8 + e;
                row[e] = (k < seg.r && 8 * c < seg.lines) ? load8_narrow(seg.src, seg.dtype, (int64_t)k * seg.lines + 8 * c) : zero;
            }
            const int64_t base = (c >> 5) * 8 * KS * 64 + (kg >> 1) * 64 + (kg & 1) * 32 + (c & 31);   // column T: + T * KS * 64
            dst[base + 0 * KS * 64] = column_of<0>(row);
            dst[base + 1 * KS * 64] = column_of<1>(row);
            dst[base + 2 * KS * 64] = column_of<2>(row);
            dst[base + 3 * KS * 64] = column_of<3>(row);
            dst[base + 4 * KS * 64] = column_of<4>(row);
            dst[base + 5 * KS * 64] = column_of<5>(row);
            dst[base + 6 * KS * 64] = column_of<6>(row);
            dst[base + 7 * KS * 64] = column_of<7>(row);
        }
        return;
    }
    if (seg.layout != kPackAt && aligned && seg.r % 8 == 0) {
        // rows of B (or plain rows): a group is 8 consecutive source elements; neighbouring lanes take
        // neighbouring groups of a row, so the reads are whole cache lines
        for (int64_t g = first; g < ngroups; g += stride) {
            const int64_t line = g / groups_per_line;
            const int kg = (int)(g - line * groups_per_line);
            const u32x4 o = (line < seg.lines && 8 * kg < seg.r) ? load8_narrow(seg.src, seg.dtype, line * seg.r + 8 * kg) : zero;
            const int64_t at = seg.layout == kPackBp ? ((line >> 5) * KS + (kg >> 1)) * 64 + (kg & 1) * 32 + (line & 31)
                                                     : line * groups_per_line + kg;
            dst[at] = o;
        }
        return;
    }
    // any rank, width and alignment: element by element
    for (int64_t g = first; g < ngroups; g += stride) {
        // consecutive lanes take consecutive lines so that the strided reads of a transposed
        // A are coalesced along j
        const int64_t line = g % lines_pad;
        const int kg = (int)(g / lines_pad);
        uint32_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int k = kg * 8 + e;
            uint32_t b = 0;
            if (k < seg.r && line < seg.lines) {             // padding lines and ranks are zeros
                // A: element (k, line) of an r x lines matrix; B (and plain rows): element (line, k) of lines x r
                const int64_t idx = seg.layout == kPackAt ? (int64_t)k * seg.lines + line : line * seg.r + k;
                b = narrow1(seg.src, seg.dtype, idx);
            }
            v[e] = b;
        }
        u32x4 o;
        o.x = pack2(v[0], v[1]);
        o.y = pack2(v[2], v[3]);
        o.z = pack2(v[4], v[5]);
        o.w = pack2(v[6], v[7]);
        // where the group of line `line`, ranks 8*kg .. 8*kg+7 lives (operand order: see lora_device.h)
        int64_t at;
        if (seg.layout == kPackAt) at = (((line >> 8) * 8 + (line & 7)) * KS + (kg >> 1)) * 64 + (kg & 1) * 32 + ((line & 255) >> 3);
        else if (seg.layout == kPackBp) at = ((line >> 5) * KS + (kg >> 1)) * 64 + (kg & 1) * 32 + (line & 31);
        else at = line * groups_per_line + kg;
        dst[at] = o;
    }
}

hipError_t launch_pack(const PackBatch& batch, int nseg, hipStream_t stream) {
    if (nseg <= 0) return hipSuccess;
    int64_t max_groups = 0;
    for (int i = 0; i < nseg; ++i) {
        if (batch.seg[i].layout != kPackRows && (batch.seg[i].rp & 15)) return hipErrorInvalidValue;
        int64_t g = pack_lines_padded(batch.seg[i]) * (batch.seg[i].rp >> 3);
        max_groups = g > max_groups ? g : max_groups;
    }
    int64_t blocks = (max_groups + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 1024) blocks = 1024;
    dim3 grid((unsigned)blocks, (unsigned)nseg, 1);
    hipLaunchKernelGGL(pack_adapter_kernel, grid, dim3(256), 0, stream, batch);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Stand-in consumer: integer checksum of a slot, read `passes` times.  Grid-stride over 16-byte
// vectors with a bounded number of workgroups, reduction by shuffles and LDS, one 64-bit atomic
// per workgroup (thousands of atomics on one address would cost more than the reads).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void slot_checksum_kernel(const uint16_t* __restrict__ slot, int64_t elems,
                                                            int passes, unsigned long long* __restrict__ out) {
    const int64_t nvec = elems >> 3;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t v0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned long long sum = 0;
    for (int p = 0; p < passes; ++p) {
        for (int64_t v = v0; v < nvec; v += stride) {
            const u32x4 x = __builtin_nontemporal_load((const u32x4*)slot + v);
            sum += (x.x & 0xFFFFu) + (x.x >> 16) + (x.y & 0xFFFFu) + (x.y >> 16) + (x.z & 0xFFFFu) + (x.z >> 16) +
                   (x.w & 0xFFFFu) + (x.w >> 16);
        }
        if (v0 == 0) {                                     // ragged tail (< 8 elements), one lane
            for (int64_t i = nvec << 3; i < elems; ++i) sum += slot[i];
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned lo = __shfl_down((unsigned)(sum & 0xFFFFFFFFull), off, 64);
        const unsigned hi = __shfl_down((unsigned)(sum >> 32), off, 64);
        sum += ((unsigned long long)hi << 32) | lo;
    }
    __shared__ unsigned long long part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long total = part[0] + part[1] + part[2] + part[3];
        if (total) atomicAdd(out, total);
    }
}

hipError_t launch_slot_checksum(const void* slot, int64_t elems, int passes, void* dev_sum, hipStream_t stream) {
    if (elems <= 0) return hipSuccess;
    int64_t blocks = ((elems >> 3) + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(slot_checksum_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint16_t*)slot,
                       elems, passes, (unsigned long long*)dev_sum);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Bare in-place read-modify-write probe: the LoRA kernels' tiling with the arithmetic taken out
// ---------------------------------------------------------------------------------------
// n matrices of rows x cols 16-bit elements, back to back.  A wave owns a strip of 256 columns and
// walks down rc blocks of 32 rows; per block a lane loads 16 rows x 16 bytes (non-temporal), flips
// one bit of every word and stores them back: the memory traffic of a LoRA pass (4 bytes per
// element) and nothing else.  What this runs at is the ceiling of the in-place pass for that
// row pitch and walk length.  rows % 32 == 0 and cols % 256 == 0 (checked by the launcher).
// MODE 0: read-modify-write (above); 1: the loads alone (what is read is folded into one word that is
// stored only if it has a value no input produces, so the loads cannot be dropped); 2: the stores alone
// (a pattern of the address: the memory's previous contents are lost).
template <int MODE>
__global__ __launch_bounds__(256) void rmw_probe_kernel(uint16_t* base, int rows, int cols, int strips, int rowblocks,
                                                        int rc, long long total_items) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long per_xcd = gridDim.x >> 3;
    const long long L = (long long)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    long long item = L * 4 + wave;
    if (item >= total_items) return;
    const int rowchunks = (rowblocks + rc - 1) / rc;
    const long long per_mat = (long long)strips * rowchunks;
    const long long mat = item / per_mat;
    item -= mat * per_mat;
    const int rowchunk = (int)(item / strips), strip = (int)(item - (long long)rowchunk * strips);
    uint16_t* W = base + mat * (long long)rows * cols;
    const int rb_end = (rowchunk + 1) * rc < rowblocks ? (rowchunk + 1) * rc : rowblocks;
    const int n = lane & 31, h = lane >> 5;
    uint32_t fold = 0;
    for (int rb = rowchunk * rc; rb < rb_end; ++rb) {
        u32x4 w[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = rb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
            if constexpr (MODE != 2)
                w[v] = __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4*)(W + (long long)row * cols + strip * 256 + n * 8));
            else
                w[v] = u32x4{(uint32_t)row, (uint32_t)strip, (uint32_t)n, 0u};
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            if constexpr (MODE == 0) w[v] ^= 1u;
            if constexpr (MODE == 1) fold |= (w[v].x & w[v].y & w[v].z & w[v].w);
        }
        if constexpr (MODE != 1) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                __builtin_nontemporal_store(w[v], (__attribute__((address_space(1))) u32x4*)(W + (long long)row * cols + strip * 256 + n * 8));
            }
        }
    }
    if constexpr (MODE == 1) {
        // bf16 data never has all bits set in four words of the same position of every row: practically never taken
        if (fold == 0xFFFFFFFFu && rows < 0) ((__attribute__((address_space(1))) uint32_t*)W)[0] = fold;
    }
}

hipError_t launch_rmw_probe(void* base, int64_t rows, int64_t cols, int64_t n, int rc, int mode, hipStream_t stream) {
    if (!base || rows <= 0 || cols <= 0 || n <= 0 || rc < 1 || mode < 0 || mode > 2) return hipErrorInvalidValue;
    if (rows % 32 || cols % 256 || rows > 0x7FFFFFFF || cols > 0x7FFFFFFF || (uintptr_t)base % 16) return hipErrorInvalidValue;
    const int strips = (int)(cols / 256), rowblocks = (int)(rows / 32);
    const int64_t total = (int64_t)strips * ((rowblocks + rc - 1) / rc) * n;
    const int64_t blocks = ((total + 3) / 4 + 7) / 8 * 8;
    if (blocks > 0x7FFFFFF0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks);
    if (mode == 0) hipLaunchKernelGGL(rmw_probe_kernel<0>, grid, dim3(256), 0, stream, (uint16_t*)base, (int)rows, (int)cols, strips, rowblocks, rc, (long long)total);
    else if (mode == 1) hipLaunchKernelGGL(rmw_probe_kernel<1>, grid, dim3(256), 0, stream, (uint16_t*)base, (int)rows, (int)cols, strips, rowblocks, rc, (long long)total);
    else hipLaunchKernelGGL(rmw_probe_kernel<2>, grid, dim3(256), 0, stream, (uint16_t*)base, (int)rows, (int)cols, strips, rowblocks, rc, (long long)total);
    return hipGetLastError();
}

}  // namespace tidal
