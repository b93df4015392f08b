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
// Bare in-place read-modify-write over n matrices of rows x cols 16-bit elements in the LoRA kernels'
// tiling (256-column strips, rc blocks of 32 rows per wave); rows % 32 == 0, cols % 256 == 0.
hipError_t launch_rmw_probe(void* base, int64_t rows, int64_t cols, int64_t n, int rc, int mode, hipStream_t stream);

// ---- packing of LoRA factors ------------------------------------------------------------
enum PackLayout {
    kPackRows = 0,       // dst: lines x rp, row-major (plain conversion; A kept row-major for the unmerged apply)
    kPackAt = 1,         // src: A, r x lines; dst: A transposed in MFMA operand order, lines rounded up to 256
    kPackBp = 2          // src: B, lines x r; dst: B in MFMA operand order, lines rounded up to 32
};
struct PackSegment {
    const void* src;     // device staging, or the GPU's view of pinned host memory
    void* dst;           // device: packed bf16, ranks zero padded to rp
    int64_t lines;       // in (for A) or out (for B)
    int32_t r, rp, dtype, layout;
};
// Bytes of the packed copies: padding lines are written (zeros), so they count.
inline size_t packed_at_bytes(int64_t in, int rp) { return 2 * (size_t)((in + 255) / 256 * 256) * (size_t)rp; }
inline size_t packed_bp_bytes(int64_t out, int rp) { return 2 * (size_t)((out + 31) / 32 * 32) * (size_t)rp; }
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

// How one group is launched: which kernel, its compile-time variant, the walk length and the grid.
// Decided on the host by plan_lora_launch (plan.cpp, no HIP call), executed by the launchers below,
// reported by tidal_lora_launch_info.
enum LoraKernelKind {
    kLoraNone = 0,        // nothing to do (no targets, both ranks 0)
    kLoraMfmaReg = 1,     // lora_mfma_kernel: each wave keeps its A strip in registers
    kLoraMfmaLds = 2,     // lora_mfma_lds_kernel: the four waves of a workgroup share one A strip in LDS
    kLoraOrdered = 3      // lora_ordered_kernel: vector ALUs, k-ascending chain
};
struct LoraLaunchPlan {
    int kind;
    int ks_old, ks_new;          // padded ranks / 16: 0, 1, 2 or 4
    bool pair;                   // delta tiles produced and consumed two at a time
    bool fork;
    int rc;                      // 32-row blocks one wave walks
    int waves_per_simd;          // waves per SIMD the instantiation asks for in its launch bounds (at least)
    int strips, rowblocks;       // 256-column strips and 32-row blocks of one slot
    int blocks_per_target;       // workgroups per slot
    int64_t total_blocks;        // workgroups of the launch (before rounding up to a multiple of 8)
};
LoraLaunchPlan plan_lora_launch(const LoraGroup& g, bool ordered);
// Register-strip instantiations whose registers allow two waves per SIMD without spilling (found
// by compiling), with the delta tiles two at a time: A strips of up to 32 ranks in all, and 32 old
// + 16 new.  The kernel's launch bounds and the plan both use it.
constexpr bool two_waves_fit(int ks0, int ks1) { return ks0 + ks1 <= 2 || (ks0 == 2 && ks1 == 1); }
// Rank pairs the LDS-strip kernel is instantiated for.
constexpr bool lds_kernel_exists(int ks0, int ks1) { return (ks0 == 4 || ks1 == 4) || (ks0 == 0 || ks1 == 0); }

// Matrix-core path (default) and ordered-accumulation vector path; `plan` comes from plan_lora_launch.
hipError_t launch_lora_mfma(const LoraGroup& g, const LoraLaunchPlan& plan, hipStream_t stream);
hipError_t launch_lora_mfma_lds(const LoraGroup& g, const LoraLaunchPlan& plan, hipStream_t stream);
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
// Both steps in one launch: a workgroup per tile of tile_rows (32 or 16) token rows keeps u in LDS
// (n_tiles = tiles of that height over all entries, numbered by first[]; entries of any padded rank).
hipError_t launch_apply_fused(const ApplyLongBatch& b, int n_tiles, int tile_rows, int in, hipStream_t stream);
// Both steps with ordered accumulation (any segment length): u = bf16(A x) if shrink, else the expand.
hipError_t launch_apply_ordered(const ApplyLongBatch& b, int in, bool shrink, hipStream_t stream);
// Vector-ALU pair for the short segments.
hipError_t launch_apply_shrink_short(const ApplyShortBatch& b, int in, hipStream_t stream);
hipError_t launch_apply_expand_short(const ApplyShortBatch& b, int max_out, hipStream_t stream);

// Knobs for tuning runs (walk lengths, kernel variants).  They are read from the environment only
// in builds made with -DTIDAL_TUNING_KNOBS (TIDAL_TUNING_KNOBS=1 python -m ...build --force), in
// this one function (plan.cpp); the default build ignores the environment and every field is -1
// ("no override").
struct TuningKnobs {
    int mfma_rc;        // TIDAL_MFMA_RC: 32-row blocks per wave walk
    int mfma_lds;       // TIDAL_MFMA_LDS: 1 = LDS-strip kernel wherever it exists, 0 = never
    int mfma_pair;      // TIDAL_MFMA_PAIR: delta tiles two at a time (1) or all live (0)
    int mfma_order;     // TIDAL_MFMA_ORDER: workgroup -> tile order of the LDS-strip kernel
    int mfma_dynlds;    // TIDAL_MFMA_DYNLDS: extra LDS bytes per workgroup (limits workgroups per CU)
    int apply_ct;       // TIDAL_APPLY_CT: 32-token tiles per wave of the expand kernel
    int apply_tile_rows; // TIDAL_APPLY_TILE_ROWS: 16 or 32 token rows per workgroup of the fused prompt kernel
    int trace_host;     // TIDAL_TRACE_HOST: 1 = print the calling thread's time per HIP call and per step (host_trace.h)
    int n_up_groups;    // TIDAL_UP_GROUPS: "4,12,48" = targets per group of the grouped adapter upload, given outright
    int up_groups[8];
    int apply_two_step; // TIDAL_APPLY_TWO_STEP: 1 = prompts as two launches (shrink, expand) instead of the fused one
};
TuningKnobs tuning_knobs();

inline int padded_rank(int r) { return r <= 0 ? 0 : (r <= 16 ? 16 : (r <= 32 ? 32 : 64)); }

}  // namespace tidal
#endif
