// Host-side state of libtidal shared by the translation units behind the C ABI (tidal.cpp: templates
// and materialisation; tidal_lora.cpp: adapters, attach / swap / detach, forks; tidal_apply.cpp: the
// unmerged apply): the handle types, error reporting, and the helpers that more than one of them uses.
#pragma once
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "host_trace.h"
#include "plan.h"
#include "tidal_internal.h"

namespace tidal {

// Sets the calling thread's error text (tidal_last_error) and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

}  // namespace tidal

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = HIP_TIMED(expr);                                                           \
        if (e_ != hipSuccess)                                                                      \
            return tidal::fail(TIDAL_E_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

namespace tidal {

constexpr size_t kNoOffset = ~(size_t)0;

struct PackedTarget {
    int32_t slot;
    int32_t r, rp;
    float alpha;
    size_t at_off, bp_off;   // byte offsets of At (in x rp) and Bp (out x rp) in the adapter memory
    size_t ar_off;           // byte offset of A row-major (r x in), or kNoOffset if not kept
    bool active() const { return r > 0 && alpha != 0.0f; }
};

struct AdapterRec {
    std::vector<PackedTarget> targets;   // in the caller's order
    char* dev = nullptr;
    size_t bytes = 0;
    hipEvent_t ready = nullptr;          // resident adapters: recorded when the upload and packing are done
                                         // (owned by the tidal_adapter); NULL for the in-arena copy of a
                                         // host-pointer attach, which is uploaded on the attach's own stream
};

// Work the template has enqueued and not yet seen complete: one event per (kind, stream).  Calls
// on different streams re-record different events, so tidal_template_sync and the cross-call
// ordering cover every stream used, not only the one used last.
enum MarkKind { kMarkLoad = 0, kMarkLora = 1 };
struct StreamMark {
    hipStream_t stream;
    int kind;
    hipEvent_t ev;
    bool active;
};

struct RateModel {
    double link_bytes_per_ms = 55e6;     // host -> device, adapters' factors
    double rmw_bytes_per_ms = 6.0e9;     // in-place pass over W
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};   // upload begin / end, last merge begin / end
    bool pending = false;                // ev[] recorded, not read yet
    double up_bytes = 0.0, rmw_bytes = 0.0;
};

struct SlotState {
    int64_t rows = 0, cols = 0, elems = 0;
    bool materialised = false;
    hipEvent_t ready = nullptr;
    bool ready_recorded = false;
};

constexpr int kMaxUploadGroups = 8;

}  // namespace tidal

struct tidal_adapter {
    tidal_template* owner;
    tidal::AdapterRec rec;
    bool attached;
    // host-side shortcuts of the unmerged apply, which runs once per layer and decode step
    mutable bool upload_seen_done = false;          // rec.ready was found complete once: no more stream waits on it
    mutable std::vector<int32_t> target_of_slot;    // slot -> index into rec.targets, -1: not a target (built on first use)
};

struct tidal_template {
    tidal_config cfg;
    tidal::ArenaLayout lay;
    char* arena = nullptr;
    std::vector<tidal::SlotState> slots;

    // device-side resources, created on first use
    bool dev_ready = false;
    hipEvent_t staged_ready[2] = {nullptr, nullptr};   // copy stream: chunk is in staging[b]
    hipEvent_t staging_free[2] = {nullptr, nullptr};   // consumer: staging[b] may be overwritten
    hipEvent_t bounce_free[2] = {nullptr, nullptr};    // copy stream: pinned buffer b has been read
    hipEvent_t ev_start = nullptr, ev_copy_done = nullptr;
    std::vector<tidal::StreamMark> marks;
    hipStream_t up_stream = nullptr;                   // library-owned: adapter uploads that overlap the merge
    hipEvent_t ev_up_begin = nullptr;
    hipEvent_t ev_group_copied[tidal::kMaxUploadGroups] = {}; // up_stream: the group's factors are in the staging memory
    hipEvent_t ev_group_packed[tidal::kMaxUploadGroups] = {}; // caller's stream: ... and have been read from there again
    hipStream_t staging_stream[2] = {nullptr, nullptr};   // the stream staging_free[b] was last recorded on
    // staged chunks of earlier loads that may still be queued: one record per load that staged any
    struct LoadMark { hipEvent_t done; int64_t chunks; };
    std::vector<LoadMark> load_marks;                  // oldest first
    std::vector<hipEvent_t> load_mark_pool;
    tidal::RateModel rates;
    char* bounce[2] = {nullptr, nullptr};              // pinned host, chunk_bytes each
    bool bounce_used[2] = {false, false};
    bool staging_rec[2] = {false, false};

    // attach state
    bool attached = false;
    tidal::AdapterRec cur;                  // record of the attached adapter (device copy stays valid)
    tidal_adapter* cur_resident = nullptr;
    int cur_region = -1;             // in-arena region holding it, or -1

    tidal_stats stats = {};

    // TIDAL_FLAG_KERNEL_TIMING: (start, stop) pairs not yet folded into stats, and a free list
    struct TimedLaunch { hipEvent_t start, stop; bool lora; };
    std::vector<TimedLaunch> timed;
    std::vector<hipEvent_t> timing_pool;
};

namespace tidal {

// --- tidal.cpp -----------------------------------------------------------------------------
// Creates the template's events on first use and resolves this device's scratch address.
int ensure_device(tidal_template* t);
// Record that `stream` now carries work of this kind for the template.
int mark_done(tidal_template* t, int kind, hipStream_t stream);
// Make `stream` wait (on the GPU) for the template's outstanding work of this kind on other streams.
int wait_marks(tidal_template* t, int kind, hipStream_t stream);
int ensure_bounce(tidal_template* t, int b);
int ensure_upload_stream(tidal_template* t);
// Kernel timing: begin returns the start event (already recorded), end records the stop event.
int timing_begin(tidal_template* t, hipStream_t s, hipEvent_t* start);
int timing_end(tidal_template* t, hipStream_t s, hipEvent_t start, bool lora);
bool host_is_pinned(const void* p);
inline char* slot_ptr(const tidal_template* t, int32_t slot) { return t->arena + t->lay.slot_offset[slot]; }
// Copy of a pageable source into a pinned buffer, split among a few host threads when large.
void gather_copy(char* dst, const char* src, size_t bytes, int threads);
int gather_sources(const tidal_template* t, const tidal_src* srcs, int32_t n_src, int32_t assume_pinned,
                   std::vector<SourceInfo>* out);
// With an adapter attached, re-materialising is allowed only if it restores every merged slot.
int check_rematerialise(const tidal_template* t, const std::vector<SourceInfo>& srcs, bool* clears);
// The streaming loop.  `fuse` (optional): an adapter already packed on the device whose delta is
// added to its targets' slots while they are written (one rounding from the source).
int materialize_impl(tidal_template* t, std::vector<SourceInfo>& infos, bool clears, void* copy_stream,
                     void* compute_stream, const AdapterRec* fuse);

// --- tidal_lora.cpp ------------------------------------------------------------------------
// One in-place pass over the targeted slots: W - delta(older) + delta(newer); either may be NULL.
int launch_rmw(tidal_template* t, const AdapterRec* older, const AdapterRec* newer, hipStream_t stream);

// --- tidal_apply.cpp -----------------------------------------------------------------------
// Resolves the current device's address of the allocation-free apply's scratch array, once per device.
int resolve_scratch();

// Issues the copies of a plan and hands every staged chunk to a consumer.  Used by
// tidal_materialize (two streams, consumer = convert kernel) and by the adapter upload
// (one stream, consumer = pack kernel).
struct Pipeline {
    tidal_template* t;
    hipStream_t copy, compute;

    // pending CPU-gathered run that will go out as one DMA
    bool run = false;
    char* run_dst = nullptr;
    const char* run_src = nullptr;
    size_t run_len = 0;

    // Small runs may be fetched by a kernel instead of the copy engine (adapter uploads, where a
    // kernel on the same stream follows and the copy -> kernel hand-over would dominate).  They
    // collect here and go out in one launch per kMaxCopyRuns, at the latest in copies_done().
    bool kernel_copy = false;
    size_t kernel_copy_max = kKernelCopyMax;
    CopyBatch kbatch;
    int kruns = 0;
    int64_t paced_chunks = 0;       // staged chunks still to come for which the host stays two ahead of the GPU (see acquire)
    int64_t staged_total = 0;       // staged chunks of this load

    int flush_kernel_copies() {
        if (kruns == 0) return TIDAL_OK;
        const int n = kruns;
        kruns = 0;
        HIP_TRY(launch_copy_from_host(kbatch, n, copy));
        return TIDAL_OK;
    }

    int flush() {
        if (!run) return TIDAL_OK;
        run = false;
        t->stats.h2d_copies++;
        if (kernel_copy && run_len <= kernel_copy_max && (uintptr_t)run_src % 16 == 0 && (uintptr_t)run_dst % 16 == 0) {
            void* view = nullptr;            // the GPU's address for this pinned host memory
            if (HIP_TIMED(hipHostGetDevicePointer(&view, const_cast<char*>(run_src), 0)) == hipSuccess && view &&
                (uintptr_t)view % 16 == 0) {
                kbatch.run[kruns++] = CopyRun{view, run_dst, (uint64_t)run_len};
                return kruns == kMaxCopyRuns ? flush_kernel_copies() : TIDAL_OK;
            }
            (void)hipGetLastError();         // not mapped: the copy engine takes it
        }
        HIP_TRY(hipMemcpyAsync(run_dst, run_src, run_len, hipMemcpyHostToDevice, copy));
        return TIDAL_OK;
    }

    // Copy one piece of `bytes` host bytes to device address dst; gathered pieces pass through
    // pinned buffer b at buf_off first.  Consecutive pieces whose source and destination both
    // continue where the previous one ended go out as one DMA (tensor merging, Sec. 6): that is
    // the case for CPU-gathered pieces by construction, and for caller memory whenever tensors
    // sit back to back in a pinned pool.
    int put(bool gathered, int b, int64_t buf_off, const char* host, size_t bytes, char* dst) {
        t->stats.h2d_bytes += bytes;
        const char* src = host;
        size_t slack = 0;               // alignment gap that may be copied along
        if (gathered) {
            char* stage = t->bounce[b] + buf_off;
            gather_copy(stage, host, bytes, t->cfg.gather_threads);
            t->stats.gathered_bytes += bytes;
            src = stage;
            slack = kSlotAlign - 1;     // gaps inside the library's own buffers only ever land in padding
        }
        if (run && !(t->cfg.flags & TIDAL_FLAG_NO_COPY_MERGE) && src >= run_src && dst >= run_dst &&
            (size_t)(src - run_src) == (size_t)(dst - run_dst) &&
            (size_t)(src - run_src) >= run_len && (size_t)(src - run_src) - run_len <= slack &&
            run_len + bytes <= ((size_t)1 << 30)) {
            run_len = (size_t)(src - run_src) + bytes;
            return TIDAL_OK;
        }
        int rc = flush();
        if (rc) return rc;
        run = true;
        run_dst = dst;
        run_src = src;
        run_len = bytes;
        return TIDAL_OK;
    }

    // Before the first use of the buffers of chunk parity b.
    int acquire(int b, bool need_bounce, bool need_staging) {
        if (need_bounce) {
            int rc = ensure_bounce(t, b);
            if (rc) return rc;
            if (t->bounce_used[b]) HIP_TRY(hipEventSynchronize(t->bounce_free[b]));
        }
        if (need_staging) {
            // Host-side pacing.  Enqueued in one burst, a load of a few hundred chunks runs as fast
            // as one whose caller stays two chunks ahead of the GPU; many more queued cross-stream
            // waits, or a host that trails the GPU by more than a few chunks while it enqueues,
            // slow every copy down (measured: 8 chunks ahead -5 %, 32 ahead -12 %).  So: two
            // chunks ahead until at most chunks_ahead chunks remain, the rest in one burst.
            if (paced_chunks > 0 && t->staging_rec[b]) HIP_TRY(hipEventSynchronize(t->staging_free[b]));
            if (paced_chunks > 0) --paced_chunks;
            if (t->staging_rec[b]) HIP_TRY(hipStreamWaitEvent(copy, t->staging_free[b], 0));
        }
        return TIDAL_OK;
    }

    // After the last copy of a chunk has been issued.
    int copies_done(int b, bool used_bounce, bool used_staging) {
        int rc = flush();
        if (rc) return rc;
        rc = flush_kernel_copies();
        if (rc) return rc;
        if (used_bounce) {
            HIP_TRY(hipEventRecord(t->bounce_free[b], copy));
            t->bounce_used[b] = true;
        }
        if (used_staging && copy != compute) {
            HIP_TRY(hipEventRecord(t->staged_ready[b], copy));
            HIP_TRY(hipStreamWaitEvent(compute, t->staged_ready[b], 0));
        }
        return TIDAL_OK;
    }

    // After the consumer kernel of a chunk has been launched.
    int consumed(int b) {
        HIP_TRY(hipEventRecord(t->staging_free[b], compute));
        t->staging_rec[b] = true;
        t->staging_stream[b] = compute;
        t->stats.chunks++;
        return TIDAL_OK;
    }
};

}  // namespace tidal
