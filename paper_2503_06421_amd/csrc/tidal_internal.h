// Internal declarations shared by the host code and the kernels of libtidal.
// Nothing here is part of the C ABI.
#ifndef TIDAL_INTERNAL_H_
#define TIDAL_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

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
constexpr int kMaxPackSeg = 96;   // 40 bytes each in the kernel arguments; fewer, larger chunks: every
                                  // copy -> pack hand-over costs tens of microseconds of bubble
struct PackBatch { PackSegment seg[kMaxPackSeg]; };

hipError_t launch_pack(const PackBatch& batch, int nseg, hipStream_t stream);
// Copies from pinned host memory (given by its device-side address) by a kernel instead of the
// copy engine; all addresses 16-byte aligned.  Pays below a few MiB per run when a kernel follows.
struct CopyRun {
    const void* src;     // device-side address of pinned host memory
    void* dst;           // device
    uint64_t bytes;
};
constexpr int kMaxCopyRuns = 64;
struct CopyBatch { CopyRun run[kMaxCopyRuns]; };                  // 1536 bytes of kernel arguments
hipError_t launch_copy_from_host(const CopyBatch& batch, int nrun, hipStream_t stream);
constexpr size_t kKernelCopyMax = (size_t)2 << 20;

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
// Everything a launch needs travels in its kernel arguments (4 KB), in two formats:
//
// Prompts (segments of more than kApplyShortRows tokens) are few and long.  Their waves are
// short-lived (one tile each), so the chain of dependent reads in front of the first data load
// counts: one self-contained entry per (segment, target slot), found with one search.  Work
// units -- 32-token tiles for the shrink, chunks of one to kApplyChunkTiles tiles for the expand
// -- are numbered entry by entry; first[k] is entry k's first unit (INT32_MAX past the last
// entry) and a wave counts the entries <= its unit: independent reads of a compact array instead
// of a bisection.
struct ApplyLongEntry {
    const uint16_t* Ar;      // r x in bf16, A row-major
    const uint16_t* Bp;      // out x rp bf16, zero padded
    uint16_t* y;             // this slot's output: n_tokens x out
    int32_t t0, t1;          // token rows [t0, t1)
    float s;                 // alpha / r
    int32_t r, rp;           // true and padded rank
    int32_t out;
    uint32_t u_tok;          // first token row of this slot's part of the workspace
    int32_t pad_;
};
constexpr int kMaxApplyLong = 64;
struct ApplyLongBatch {
    const uint16_t* x;       // n_tokens x in, shared by all slots
    uint16_t* u;             // workspace: an entry's rows start at u + (u_tok + t0) * kApplyRankStride, pitch rp
    int32_t n, pad_;
    int32_t first[kMaxApplyLong];
    ApplyLongEntry e[kMaxApplyLong];         // 3584 bytes
};
// Decode steps (segments of at most kApplyShortRows tokens) are many and tiny: three small
// tables, so that 256 requests on up to 4 slots are one launch -- the slots (output pointer and
// width), the factors of every (adapter, slot) pair in use (offsets in 256-byte units from the
// lowest adapter address: adapters are separate allocations) and the segments (first token, row
// count and the index of their adapter's first factor entry; its other slots follow).
struct ApplySlot {
    uint16_t* y;             // n_tokens x out
    int32_t out;
    uint32_t u_tok;
};
struct ApplyFactor {
    uint32_t ar, bp;         // A row-major (r x in) and B (out x rp, zero padded)
    float s;                 // alpha / r
    uint16_t r, rp;          // true and padded rank; r = 0: nothing to do for this pair
};
struct ApplyShortSeg {
    int32_t t0;
    uint16_t rows;           // 1 .. kApplyShortRows
    uint16_t fac;            // factor entry of (adapter, slot 0)
};
constexpr int kMaxApplyShort = 256;
constexpr int kMaxApplyFactors = 96;
constexpr int kMaxApplySlots = 4;
struct ApplyShortBatch {
    const uint16_t* x;
    uint16_t* u;
    const char* adapter_base;
    int32_t n_segs, n_slots;
    ApplySlot slot[kMaxApplySlots];          //   64 bytes
    ApplyShortSeg seg[kMaxApplyShort];       // 2048
    ApplyFactor fac[kMaxApplyFactors];       // 1536
};
static_assert(sizeof(ApplyLongBatch) <= 3900 && sizeof(ApplyShortBatch) <= 3900, "kernel arguments are limited to 4 KB");
constexpr int kApplyRankStride = 64;   // workspace elements reserved per token and slot
constexpr int kApplyChunkTiles = 4;    // most 32-token tiles a wave of the expand kernel walks per strip
constexpr int kApplyShortRows = 4;     // segments up to this many tokens take the vector-ALU kernels
// Matrix-core pair: u = bf16(A x) (n_tiles = 32-token tiles over all entries), then y += s * B u
// (n_chunks = chunks over all entries; rp = the padded rank all entries of the launch have).
hipError_t launch_apply_shrink(const ApplyLongBatch& b, int n_tiles, int in, hipStream_t stream);
hipError_t launch_apply_expand(const ApplyLongBatch& b, int n_chunks, int chunk_tiles, int max_out, int rp, hipStream_t stream);
// Both steps with ordered accumulation (any segment length): u = bf16(A x) if shrink, else the expand.
hipError_t launch_apply_ordered(const ApplyLongBatch& b, int in, bool shrink, hipStream_t stream);
// Vector-ALU pair for the short segments.
hipError_t launch_apply_shrink_short(const ApplyShortBatch& b, int in, hipStream_t stream);
hipError_t launch_apply_expand_short(const ApplyShortBatch& b, int max_out, hipStream_t stream);

// Knobs for tuning runs (walk lengths, kernel variants).  They are read from the environment only
// in builds made with -DTIDAL_TUNING_KNOBS (TIDAL_TUNING_KNOBS=1 python -m ...build --force); the
// default build ignores the environment and has no code path that depends on it.
inline const char* tuning_knob(const char* name) {
#ifdef TIDAL_TUNING_KNOBS
    return getenv(name);
#else
    (void)name;
    return nullptr;
#endif
}

inline int padded_rank(int r) { return r <= 0 ? 0 : (r <= 16 ? 16 : (r <= 32 ? 32 : 64)); }

}  // namespace tidal
#endif
