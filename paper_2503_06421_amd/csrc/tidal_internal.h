// Internal declarations shared by the host code and the kernels of libtidal.
// Nothing here is part of the C ABI.
#ifndef TIDAL_INTERNAL_H_
#define TIDAL_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tidal.h"

namespace tidal {

// ---- conversion of a staged chunk -----------------------------------------------------
struct ConvertSegment {
    const void* src;   // device, 16-byte aligned (inside a staging buffer)
    void* dst;         // device, 16-byte aligned (inside a slot)
    int64_t elems;
    int32_t dtype;
    int32_t pad_;
};
constexpr int kMaxConvertSeg = 32;
struct ConvertBatch { ConvertSegment seg[kMaxConvertSeg]; };

hipError_t launch_convert(const ConvertBatch& batch, int nseg, hipStream_t stream);
hipError_t launch_slot_checksum(const void* slot, int64_t elems, int passes, void* dev_sum, hipStream_t stream);

// ---- packing of LoRA factors ------------------------------------------------------------
struct PackSegment {
    const void* src;     // device staging: A (r x lines, transposed = 1) or B (lines x r)
    void* dst;           // device: lines x rp bf16
    int64_t lines;       // in (for A) or out (for B)
    int32_t r, rp, dtype, transposed;
};
constexpr int kMaxPackSeg = 32;
struct PackBatch { PackSegment seg[kMaxPackSeg]; };

hipError_t launch_pack(const PackBatch& batch, int nseg, hipStream_t stream);

// ---- LoRA read-modify-write ---------------------------------------------------------------
// One entry per targeted slot of a launch.  All slots of a launch share out, in and the padded
// ranks of the old and new adapter.  Addresses are 256-byte units relative to three bases (the
// arena and the memory of the two adapters), which keeps an entry at 28 bytes so that 128 of them
// travel in the kernel arguments: no table in device memory, no copy before the launch.  Larger
// groups are split; every launch still covers tens of millions of elements.
struct LoraTargetDev {
    uint32_t w;              // slot: out x in bf16, relative to w_base
    uint32_t at_old, bp_old; // in x rp_old (A transposed, zero padded) and out x rp_old, rel. to old_base
    uint32_t at_new, bp_new; // same for the new adapter, relative to new_base
    float s_old;             // already negated: W - (alpha/r) * delta_old
    float s_new;
};
constexpr int kMaxLoraTargets = 128;
constexpr size_t kLoraUnit = 256;
struct LoraBatch {
    char* w_base;
    const char* old_base;
    const char* new_base;
    LoraTargetDev t[kMaxLoraTargets];     // 3584 bytes
};

struct LoraGroup {
    const LoraBatch* batch;      // host; copied into the kernel arguments at launch
    int32_t n_targets;           // <= kMaxLoraTargets
    int32_t out, in;
    int32_t r_old, r_new;        // true ranks (ordered-accumulation kernel)
    int32_t rp_old, rp_new;      // padded ranks: 0, 16, 32 or 64
    bool fork;                   // write to old_base + at_old instead of in place (rp_old must be 0)
};

// Matrix-core path (default) and ordered-accumulation vector path.
hipError_t launch_lora_mfma(const LoraGroup& g, hipStream_t stream);
hipError_t launch_lora_ordered(const LoraGroup& g, hipStream_t stream);

// ---- materialisation with the adapter folded in --------------------------------------------
// One staged piece (elements [e0, e0 + n) of a slot, in the source's dtype) of a LoRA target.
struct FusedPiece {
    const void* src;         // device staging: the piece in its host dtype (fp32 or fp16)
    uint16_t* slot;          // slot base: out x in bf16
    const uint16_t* At;      // in x rp
    const uint16_t* Bp;      // out x rp
    int64_t e0, n;
    int32_t out, in, dtype, r, rp;
    float s;                 // alpha / r
};
// slot[e] = bf16(f32(src[e - e0]) + s * (B A)[e]) for the piece; ordered: k-ascending FMA chain
hipError_t launch_convert_merge(const FusedPiece& p, bool ordered, hipStream_t stream);

// ---- unmerged adapter apply ---------------------------------------------------------------
// One entry per run of consecutive tokens that share an adapter.  Adapters live in separate
// caller-owned allocations, hence full pointers; 80 entries travel in the kernel arguments,
// batches with more segments take several launches.  Work units (32-token tiles for the shrink,
// chunks of one to kApplyChunkTiles tiles for the expand) are numbered through the launch; first[k]
// is the number of segment k's first one (INT32_MAX past the last segment).  The kernels count
// the entries <= their unit: one independent read of a compact array instead of a bisection,
// whose dependent reads of the kernel arguments would cost more than a small batch's work.
struct ApplySeg {
    const uint16_t* Ar;      // r x in bf16, A row-major
    const uint16_t* Bp;      // out x rp bf16, zero padded
    int32_t t0, t1;          // token rows [t0, t1)
    float s;                 // alpha / r
    int32_t r, rp;           // true and padded rank
    int32_t pad_;
};
constexpr int kMaxApplySegs = 80;
constexpr int kApplyRankStride = 64;   // workspace elements reserved per token
constexpr int kApplyChunkTiles = 4;    // most 32-token tiles a wave of the expand kernel walks per strip
constexpr int kApplyShortRows = 4;     // segments up to this many tokens take the vector-ALU expand
struct ApplyBatch {
    const uint16_t* x;       // n_tokens x in
    uint16_t* y;             // n_tokens x out
    uint16_t* u;             // workspace: token t's rank-space row at u + t0 * kApplyRankStride + (t - t0) * rp
    int32_t n_segs, pad_;
    int32_t first[kMaxApplySegs];
    ApplySeg seg[kMaxApplySegs];   // 3200 bytes
};
// Segments longer than kApplyShortRows tokens take the matrix-core kernels: u = bf16(A x)
// (n_tiles = total 32-token tiles), then y += s * B u (n_chunks = total chunks; all segments of
// that launch share the padded rank rp).  Shorter ones take the vector-ALU pair.
hipError_t launch_apply_shrink(const ApplyBatch& b, int n_tiles, int in, hipStream_t stream);
hipError_t launch_apply_expand(const ApplyBatch& b, int n_chunks, int chunk_tiles, int out, int rp, hipStream_t stream);
hipError_t launch_apply_shrink_short(const ApplyBatch& b, int in, hipStream_t stream);
hipError_t launch_apply_expand_short(const ApplyBatch& b, int out, hipStream_t stream);

inline int padded_rank(int r) { return r <= 0 ? 0 : (r <= 16 ? 16 : (r <= 32 ? 32 : 64)); }

}  // namespace tidal
#endif
