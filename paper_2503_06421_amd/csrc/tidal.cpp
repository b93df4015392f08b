// libtidal host side: the C ABI, argument validation, the attach/swap state machine and
// the two-stream staging pipeline.  All arithmetic on tensor data happens in the kernels
// (convert_kernels.hip, lora_kernels.hip); this file only moves bytes and launches.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <tuple>
#include <vector>

#include "host_trace.h"
#include "plan.h"
#include "tidal_internal.h"

using namespace tidal;

// ---------------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = HIP_TIMED(expr);                                                           \
        if (e_ != hipSuccess)                                                                      \
            return fail(TIDAL_E_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    } while (0)

// ---------------------------------------------------------------------------------------
// handles
// ---------------------------------------------------------------------------------------
namespace {

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

}  // namespace

constexpr int kMaxUploadGroups = 8;

// ---------------------------------------------------------------------------------------
// scratch memory of the allocation-free apply (tidal_lora_apply_static)
// ---------------------------------------------------------------------------------------
// The rank-space intermediate u = bf16(A x) of the unmerged apply normally lives in a workspace the
// caller allocates.  Callers that cannot allocate get it from this array instead: 128 bytes per
// token row, kStaticApplyTokens rows, 2 MiB that every GPU the library runs on holds until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels
// and copies get the per-device address that call returns.
constexpr int32_t kStaticApplyTokens = 16384;
constexpr size_t kStaticScratchBytes = (size_t)kStaticApplyTokens * kApplyRankStride * 2;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices] = {};          // per device: each GPU has its own copy of the array

// Set-up step, run with the device current that the calling template works on: resolves this
// device's address of the scratch array once.
static int resolve_scratch() {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(TIDAL_E_HIP, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(TIDAL_E_HIP, "hipGetSymbolAddress returned no address for the scratch array");
        g_scratch_ptr[dev] = p;
    }
    return TIDAL_OK;
}

struct tidal_adapter {
    tidal_template* owner;
    AdapterRec rec;
    bool attached;
    // host-side shortcuts of the unmerged apply, which runs once per layer and decode step
    mutable bool upload_seen_done = false;          // rec.ready was found complete once: no more stream waits on it
    mutable std::vector<int32_t> target_of_slot;    // slot -> index into rec.targets, -1: not a target (built on first use)
};

struct tidal_template {
    tidal_config cfg;
    ArenaLayout lay;
    char* arena = nullptr;
    std::vector<SlotState> slots;

    // device-side resources, created on first use
    bool dev_ready = false;
    hipEvent_t staged_ready[2] = {nullptr, nullptr};   // copy stream: chunk is in staging[b]
    hipEvent_t staging_free[2] = {nullptr, nullptr};   // consumer: staging[b] may be overwritten
    hipEvent_t bounce_free[2] = {nullptr, nullptr};    // copy stream: pinned buffer b has been read
    hipEvent_t ev_start = nullptr, ev_copy_done = nullptr;
    std::vector<StreamMark> marks;
    hipStream_t up_stream = nullptr;                   // library-owned: adapter uploads that overlap the merge
    hipEvent_t ev_up_begin = nullptr;
    hipEvent_t ev_group_copied[kMaxUploadGroups] = {}; // up_stream: the group's factors are in the staging memory
    hipEvent_t ev_group_packed[kMaxUploadGroups] = {}; // caller's stream: ... and have been read from there again
    hipStream_t staging_stream[2] = {nullptr, nullptr};   // the stream staging_free[b] was last recorded on
    // staged chunks of earlier loads that may still be queued: one record per load that staged any
    struct LoadMark { hipEvent_t done; int64_t chunks; };
    std::vector<LoadMark> load_marks;                  // oldest first
    std::vector<hipEvent_t> load_mark_pool;
    RateModel rates;
    char* bounce[2] = {nullptr, nullptr};              // pinned host, chunk_bytes each
    bool bounce_used[2] = {false, false};
    bool staging_rec[2] = {false, false};

    // attach state
    bool attached = false;
    AdapterRec cur;                  // record of the attached adapter (device copy stays valid)
    tidal_adapter* cur_resident = nullptr;
    int cur_region = -1;             // in-arena region holding it, or -1

    tidal_stats stats = {};

    // TIDAL_FLAG_KERNEL_TIMING: (start, stop) pairs not yet folded into stats, and a free list
    struct TimedLaunch { hipEvent_t start, stop; bool lora; };
    std::vector<TimedLaunch> timed;
    std::vector<hipEvent_t> timing_pool;
};

// ---------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------
static int ensure_device(tidal_template* t) {
    if (t->dev_ready) return TIDAL_OK;
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return fail(TIDAL_E_HIP, "no HIP device available (%s)", hipGetErrorString(e));
    }
    const unsigned flags = hipEventDisableTiming;
    for (int b = 0; b < 2; ++b) {
        HIP_TRY(hipEventCreateWithFlags(&t->staged_ready[b], flags));
        HIP_TRY(hipEventCreateWithFlags(&t->staging_free[b], flags));
        HIP_TRY(hipEventCreateWithFlags(&t->bounce_free[b], flags));
    }
    HIP_TRY(hipEventCreateWithFlags(&t->ev_start, flags));
    HIP_TRY(hipEventCreateWithFlags(&t->ev_copy_done, flags));
    int rc = resolve_scratch();
    if (rc) return rc;
    t->dev_ready = true;
    return TIDAL_OK;
}

// Record that `stream` now carries work of this kind for the template.
static int mark_done(tidal_template* t, int kind, hipStream_t stream) {
    for (StreamMark& m : t->marks)
        if (m.stream == stream && m.kind == kind) {
            HIP_TRY(hipEventRecord(m.ev, stream));
            m.active = true;
            return TIDAL_OK;
        }
    StreamMark m{stream, kind, nullptr, true};
    HIP_TRY(hipEventCreateWithFlags(&m.ev, hipEventDisableTiming));
    HIP_TRY(hipEventRecord(m.ev, stream));
    t->marks.push_back(m);
    return TIDAL_OK;
}

// Make `stream` wait (on the GPU) for the template's outstanding work of this kind on other streams.
static int wait_marks(tidal_template* t, int kind, hipStream_t stream) {
    for (const StreamMark& m : t->marks)
        if (m.active && m.kind == kind && m.stream != stream) HIP_TRY(hipStreamWaitEvent(stream, m.ev, 0));
    return TIDAL_OK;
}

static int ensure_bounce(tidal_template* t, int b) {
    if (!t->bounce[b]) HIP_TRY(hipHostMalloc((void**)&t->bounce[b], t->cfg.chunk_bytes, hipHostMallocDefault));
    return TIDAL_OK;
}

static int ensure_upload_stream(tidal_template* t) {
    if (t->up_stream) return TIDAL_OK;
    HIP_TRY(hipStreamCreateWithFlags(&t->up_stream, hipStreamNonBlocking));      // default priority
    HIP_TRY(hipEventCreateWithFlags(&t->ev_up_begin, hipEventDisableTiming));
    for (int g = 0; g < kMaxUploadGroups; ++g) {
        HIP_TRY(hipEventCreateWithFlags(&t->ev_group_copied[g], hipEventDisableTiming));
        HIP_TRY(hipEventCreateWithFlags(&t->ev_group_packed[g], hipEventDisableTiming));
    }
    for (int k = 0; k < 4; ++k) HIP_TRY(hipEventCreate(&t->rates.ev[k]));
    return TIDAL_OK;
}

// Kernel timing: begin returns the start event (already recorded), end records the stop event.
static int timing_begin(tidal_template* t, hipStream_t s, hipEvent_t* start) {
    *start = nullptr;
    if (!(t->cfg.flags & TIDAL_FLAG_KERNEL_TIMING)) return TIDAL_OK;
    if (t->timing_pool.empty()) {
        HIP_TRY(hipEventCreate(start));
    } else {
        *start = t->timing_pool.back();
        t->timing_pool.pop_back();
    }
    HIP_TRY(hipEventRecord(*start, s));
    return TIDAL_OK;
}

static int timing_end(tidal_template* t, hipStream_t s, hipEvent_t start, bool lora) {
    if (!start) return TIDAL_OK;
    hipEvent_t stop = nullptr;
    if (t->timing_pool.empty()) {
        HIP_TRY(hipEventCreate(&stop));
    } else {
        stop = t->timing_pool.back();
        t->timing_pool.pop_back();
    }
    HIP_TRY(hipEventRecord(stop, s));
    t->timed.push_back(tidal_template::TimedLaunch{start, stop, lora});
    return TIDAL_OK;
}

static int timing_drain(tidal_template* t) {
    for (auto& tl : t->timed) {
        HIP_TRY(hipEventSynchronize(tl.stop));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, tl.start, tl.stop));
        (tl.lora ? t->stats.lora_kernel_ms : t->stats.convert_kernel_ms) += (double)ms;
        t->timing_pool.push_back(tl.start);
        t->timing_pool.push_back(tl.stop);
    }
    t->timed.clear();
    return TIDAL_OK;
}

static bool host_is_pinned(const void* p) {
    hipPointerAttribute_t attr;
    hipError_t e = HIP_TIMED(hipPointerGetAttributes(&attr, p));
    if (e != hipSuccess) {
        (void)hipGetLastError();   // plain malloc'ed memory is reported as an error, not a type
        return false;
    }
    return attr.type == hipMemoryTypeHost;
}

static inline char* slot_ptr(const tidal_template* t, int32_t slot) { return t->arena + t->lay.slot_offset[slot]; }

// ---------------------------------------------------------------------------------------
// configuration, creation
// ---------------------------------------------------------------------------------------
extern "C" int tidal_config_default(tidal_config* cfg) {
    if (!cfg) return fail(TIDAL_E_INVAL, "cfg is NULL");
    const char* msg = "";
    normalise_config(nullptr, cfg, &msg);
    return TIDAL_OK;
}

extern "C" size_t tidal_template_required_bytes(const tidal_slot_desc* slots, int32_t n, const tidal_config* cfg) {
    if ((!slots && n > 0) || n < 0) return 0;
    tidal_config c;
    const char* msg = "";
    if (!normalise_config(cfg, &c, &msg)) return 0;
    ArenaLayout lay;
    if (!layout_arena(slots, n, c, &lay)) return 0;
    return lay.total;
}

extern "C" int tidal_template_create(const tidal_slot_desc* slots, int32_t n, void* dev_arena, size_t arena_bytes,
                                     const tidal_config* cfg, tidal_template** out) {
    if (!out) return fail(TIDAL_E_INVAL, "out is NULL");
    *out = nullptr;
    if (n < 0 || (!slots && n > 0)) return fail(TIDAL_E_INVAL, "bad slot list (n=%d)", n);
    if (!dev_arena) return fail(TIDAL_E_INVAL, "dev_arena is NULL");
    if ((uintptr_t)dev_arena % kSlotAlign) return fail(TIDAL_E_INVAL, "dev_arena is not 256-byte aligned");
    tidal_config c;
    const char* msg = "";
    if (!normalise_config(cfg, &c, &msg)) return fail(TIDAL_E_INVAL, "config: %s", msg);
    tidal_template* t = new (std::nothrow) tidal_template();
    if (!t) return fail(TIDAL_E_NOMEM, "out of host memory");
    t->cfg = c;
    if (!layout_arena(slots, n, c, &t->lay)) {
        delete t;
        return fail(TIDAL_E_INVAL, "slot with negative or oversized shape");
    }
    if (t->lay.total > arena_bytes) {
        size_t need = t->lay.total;
        delete t;
        return fail(TIDAL_E_NOMEM, "arena too small: need %zu bytes, got %zu", need, arena_bytes);
    }
    t->arena = (char*)dev_arena;
    t->slots.resize((size_t)n);
    for (int32_t i = 0; i < n; ++i) {
        t->slots[i].rows = slots[i].rows;
        t->slots[i].cols = slots[i].cols;
        t->slots[i].elems = slots[i].rows * slots[i].cols;
    }
    *out = t;
    return TIDAL_OK;
}

extern "C" int tidal_template_slot_ptr(const tidal_template* t, int32_t slot, void** dev_ptr, size_t* bytes) {
    if (!t || !dev_ptr) return fail(TIDAL_E_INVAL, "NULL argument");
    if (slot < 0 || slot >= (int32_t)t->slots.size()) return fail(TIDAL_E_INVAL, "slot %d out of range", slot);
    *dev_ptr = slot_ptr(t, slot);
    if (bytes) *bytes = 2 * (size_t)t->slots[slot].elems;
    return TIDAL_OK;
}

// ---------------------------------------------------------------------------------------
// materialisation
// ---------------------------------------------------------------------------------------
// Copy of a pageable source into the pinned buffer.  One host thread moves about 27 GB/s here,
// half of what the link carries, so large pieces are split among a few threads (started per
// piece: tens of microseconds against the millisecond the piece takes).
static void gather_copy(char* dst, const char* src, size_t bytes, int threads) {
    constexpr size_t kSplitFrom = (size_t)8 << 20;
    if (threads <= 1 || bytes < kSplitFrom) {
        memcpy(dst, src, bytes);
        return;
    }
    const size_t part = (bytes / threads + 4095) & ~(size_t)4095;
    std::vector<std::thread> pool;
    for (int k = 1; k < threads; ++k) {
        const size_t o = (size_t)k * part;
        if (o >= bytes) break;
        const size_t n = std::min(part, bytes - o);
        pool.emplace_back([=] { memcpy(dst + o, src + o, n); });
    }
    memcpy(dst, src, std::min(part, bytes));
    for (std::thread& th : pool) th.join();
}

static int gather_sources(const tidal_template* t, const tidal_src* srcs, int32_t n_src, int32_t assume_pinned,
                          std::vector<SourceInfo>* out) {
    if (!t) return fail(TIDAL_E_INVAL, "template is NULL");
    if (n_src < 0 || (!srcs && n_src > 0)) return fail(TIDAL_E_INVAL, "bad source list (n=%d)", n_src);
    std::vector<char> seen(t->slots.size(), 0);
    out->clear();
    out->reserve((size_t)n_src);
    for (int32_t i = 0; i < n_src; ++i) {
        const tidal_src& s = srcs[i];
        if (s.slot < 0 || s.slot >= (int32_t)t->slots.size())
            return fail(TIDAL_E_INVAL, "source %d: slot %d out of range", i, s.slot);
        if (!dtype_ok(s.dtype)) return fail(TIDAL_E_INVAL, "source %d: unknown dtype %d", i, s.dtype);
        if (seen[s.slot]) return fail(TIDAL_E_INVAL, "source %d: slot %d given twice", i, s.slot);
        seen[s.slot] = 1;
        const int64_t elems = t->slots[s.slot].elems;
        if (!s.host && elems > 0) return fail(TIDAL_E_INVAL, "source %d: host pointer is NULL", i);
        bool pinned = assume_pinned > 0;
        if (assume_pinned < 0) pinned = elems > 0 && host_is_pinned(s.host);
        out->push_back(SourceInfo{s.slot, s.dtype, (const char*)s.host, elems, pinned});
    }
    return TIDAL_OK;
}

// With an adapter attached, re-materialising is allowed only if it restores every merged slot.
static int check_rematerialise(const tidal_template* t, const std::vector<SourceInfo>& srcs, bool* clears) {
    *clears = false;
    if (!t->attached) return TIDAL_OK;
    std::vector<char> covered(t->slots.size(), 0);
    for (const SourceInfo& s : srcs) covered[s.slot] = 1;
    int hit = 0, total = 0;
    for (const PackedTarget& p : t->cur.targets) {
        if (!p.active()) continue;
        ++total;
        hit += covered[p.slot];
    }
    if (hit == 0) return TIDAL_OK;
    if (hit != total)
        return fail(TIDAL_E_STATE, "materialize covers %d of the %d slots the attached adapter is merged into", hit, total);
    *clears = true;
    return TIDAL_OK;
}

extern "C" int32_t tidal_materialize_plan(tidal_template* t, const tidal_src* srcs, int32_t n_src,
                                          int32_t assume_pinned, tidal_copy_piece* out, int32_t cap) {
    std::vector<SourceInfo> infos;
    int rc = gather_sources(t, srcs, n_src, assume_pinned, &infos);
    if (rc) return rc;
    if (cap < 0 || (!out && cap > 0)) return fail(TIDAL_E_INVAL, "bad output buffer");
    std::vector<Piece> plan;
    plan_copies(infos, t->cfg, kMaxConvertSeg, &plan);
    for (size_t i = 0; i < plan.size() && (int32_t)i < cap; ++i) {
        const Piece& p = plan[i];
        out[i].chunk = p.chunk;
        out[i].slot = p.slot;
        out[i].elem_offset = p.elem_offset;
        out[i].elems = p.elems;
        out[i].src_bytes = p.src_bytes;
        out[i].staging_offset = p.staged ? p.buf_offset : -1;
        out[i].gathered = p.gathered ? 1 : 0;
        out[i].reserved = 0;
    }
    return (int32_t)plan.size();
}

namespace {

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

}  // namespace

static int launch_rmw(tidal_template* t, const AdapterRec* older, const AdapterRec* newer, hipStream_t stream);

// The streaming loop.  `fuse` (optional): an adapter already packed on the device whose delta is
// added to its targets' slots while they are written (one rounding from the source).
static int materialize_impl(tidal_template* t, std::vector<SourceInfo>& infos, bool clears, void* copy_stream,
                            void* compute_stream, const AdapterRec* fuse) {
    if (infos.empty()) return TIDAL_OK;
    int rc = ensure_device(t);
    if (rc) return rc;
    for (SourceInfo& s : infos) s.pinned = s.elems > 0 && host_is_pinned(s.host);
    std::vector<const PackedTarget*> fused_of(t->slots.size(), nullptr);
    if (fuse)
        for (const PackedTarget& p : fuse->targets)
            if (p.active() && t->slots[p.slot].elems > 0) fused_of[p.slot] = &p;
    const bool ordered = (t->cfg.flags & TIDAL_FLAG_ORDERED_ACCUM) != 0;
    AdapterRec direct;                 // targets whose bf16 source goes straight into the slot: merged afterwards
    if (fuse) direct.dev = fuse->dev;

    std::vector<Piece> plan;
    plan_copies(infos, t->cfg, kMaxConvertSeg, &plan);

    Pipeline pl{t, (hipStream_t)copy_stream, (hipStream_t)compute_stream};
    if (!(t->cfg.flags & TIDAL_FLAG_ASYNC_ENQUEUE)) {
        int64_t staged_chunks = 0;
        int32_t last = -1;
        for (const Piece& p : plan)
            if (p.staged && p.chunk != last) {
                ++staged_chunks;
                last = p.chunk;
            }
        // the burst budget is what earlier loads, as far as they are still in flight, have left of it
        int64_t queued = 0;
        while (!t->load_marks.empty() && hipEventQuery(t->load_marks.front().done) == hipSuccess) {
            t->load_mark_pool.push_back(t->load_marks.front().done);
            t->load_marks.erase(t->load_marks.begin());
        }
        (void)hipGetLastError();                           // hipErrorNotReady is no error here
        for (const auto& m : t->load_marks) queued += m.chunks;
        const int64_t budget = std::max<int64_t>(0, (int64_t)t->cfg.chunks_ahead - queued);
        pl.paced_chunks = std::max<int64_t>(0, staged_chunks - budget);
        pl.staged_total = staged_chunks;
    }
    // LoRA kernels of this template may have run on another stream: order after them
    rc = wait_marks(t, kMarkLora, pl.compute);
    if (rc) return rc;
    if (pl.copy != pl.compute) {
        rc = wait_marks(t, kMarkLora, pl.copy);
        if (rc) return rc;
        for (const StreamMark& m : t->marks)             // LoRA work on the compute stream itself
            if (m.active && m.kind == kMarkLora && m.stream == pl.compute) HIP_TRY(hipStreamWaitEvent(pl.copy, m.ev, 0));
    }
    // copies may write slots that earlier work on the compute stream still reads
    if (pl.copy != pl.compute) {
        HIP_TRY(hipEventRecord(t->ev_start, pl.compute));
        HIP_TRY(hipStreamWaitEvent(pl.copy, t->ev_start, 0));
    }
    const bool slot_events = (t->cfg.flags & TIDAL_FLAG_SLOT_EVENTS) != 0;

    size_t i = 0;
    while (i < plan.size()) {
        const int32_t chunk = plan[i].chunk;
        const int b = chunk & 1;
        size_t j = i;
        bool need_bounce = false, need_staging = false;
        while (j < plan.size() && plan[j].chunk == chunk) {
            need_bounce |= plan[j].gathered;
            need_staging |= plan[j].staged;
            ++j;
        }
        rc = pl.acquire(b, need_bounce, need_staging);
        if (rc) return rc;
        ConvertBatch batch;
        int nseg = 0;
        std::vector<FusedPiece> fused;
        for (size_t k = i; k < j; ++k) {
            const Piece& p = plan[k];
            char* slot_dst = slot_ptr(t, p.slot) + 2 * p.elem_offset;
            char* dst = p.staged ? t->arena + t->lay.staging[b] + p.buf_offset : slot_dst;
            rc = pl.put(p.gathered, b, p.buf_offset, p.host, (size_t)p.src_bytes, dst);
            if (rc) return rc;
            const PackedTarget* ft = fused_of[p.slot];
            if (p.staged && ft) {
                const SlotState& st = t->slots[p.slot];
                fused.push_back(FusedPiece{dst, (uint16_t*)slot_ptr(t, p.slot), (const uint16_t*)(fuse->dev + ft->at_off),
                                           (const uint16_t*)(fuse->dev + ft->bp_off), p.elem_offset, p.elems,
                                           (int32_t)st.rows, (int32_t)st.cols, p.dtype, ft->r, ft->rp,
                                           ft->alpha / (float)ft->r});
                t->stats.converted_elems += (uint64_t)p.elems;
            } else if (p.staged) {
                batch.seg[nseg++] = ConvertSegment{dst, slot_dst, p.elems, p.dtype, 0};
                t->stats.converted_elems += (uint64_t)p.elems;
            } else if (ft && p.elem_offset == 0) {
                direct.targets.push_back(*ft);
            }
        }
        rc = pl.copies_done(b, need_bounce, need_staging);
        if (rc) return rc;
        if (need_staging) {
            hipEvent_t t0;
            rc = timing_begin(t, pl.compute, &t0);
            if (rc) return rc;
            HIP_TRY(launch_convert(batch, nseg, pl.compute));
            for (const FusedPiece& fp : fused) HIP_TRY(launch_convert_merge(fp, ordered, pl.compute));
            rc = timing_end(t, pl.compute, t0, false);
            if (rc) return rc;
            rc = pl.consumed(b);
            if (rc) return rc;
        }
        if (slot_events) {
            // a slot is complete when the chunk holding its last piece is done
            for (size_t k = i; k < j; ++k) {
                const Piece& p = plan[k];
                if (p.elem_offset + p.elems != t->slots[p.slot].elems) continue;
                SlotState& s = t->slots[p.slot];
                if (!s.ready) HIP_TRY(hipEventCreateWithFlags(&s.ready, hipEventDisableTiming));
                HIP_TRY(hipEventRecord(s.ready, p.staged ? pl.compute : pl.copy));
                s.ready_recorded = true;
            }
        }
        i = j;
    }
    // completion of the compute stream implies completion of the call
    if (pl.copy != pl.compute) {
        HIP_TRY(hipEventRecord(t->ev_copy_done, pl.copy));
        HIP_TRY(hipStreamWaitEvent(pl.compute, t->ev_copy_done, 0));
    }
    rc = mark_done(t, kMarkLoad, pl.compute);
    if (rc) return rc;
    if (pl.staged_total > 0 && !(t->cfg.flags & TIDAL_FLAG_ASYNC_ENQUEUE)) {
        hipEvent_t e = nullptr;
        if (!t->load_mark_pool.empty()) {
            e = t->load_mark_pool.back();
            t->load_mark_pool.pop_back();
        } else {
            HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        }
        HIP_TRY(hipEventRecord(e, pl.compute));
        t->load_marks.push_back({e, pl.staged_total});
    }
    for (const SourceInfo& s : infos) t->slots[s.slot].materialised = true;
    if (!direct.targets.empty()) {
        // bf16 sources are exact in the slot already: the in-place merge is the same single rounding
        rc = launch_rmw(t, nullptr, &direct, pl.compute);
        if (rc) return rc;
        rc = mark_done(t, kMarkLoad, pl.compute);
        if (rc) return rc;
    }
    if (clears) {
        if (t->cur_resident) t->cur_resident->attached = false;
        t->attached = false;
        t->cur_resident = nullptr;
        t->cur_region = -1;
        t->cur.targets.clear();
    }
    return TIDAL_OK;
}

extern "C" int tidal_materialize(tidal_template* t, const tidal_src* srcs, int32_t n_src, void* copy_stream,
                                 void* compute_stream) {
    std::vector<SourceInfo> infos;
    int rc = gather_sources(t, srcs, n_src, 0, &infos);
    if (rc) return rc;
    bool clears = false;
    rc = check_rematerialise(t, infos, &clears);
    if (rc) return rc;
    return materialize_impl(t, infos, clears, copy_stream, compute_stream, nullptr);
}

extern "C" int tidal_template_slot_wait(tidal_template* t, int32_t slot, void* stream) {
    if (!t) return fail(TIDAL_E_INVAL, "template is NULL");
    if (slot < 0 || slot >= (int32_t)t->slots.size()) return fail(TIDAL_E_INVAL, "slot %d out of range", slot);
    if (!(t->cfg.flags & TIDAL_FLAG_SLOT_EVENTS)) return fail(TIDAL_E_STATE, "template was created without TIDAL_FLAG_SLOT_EVENTS");
    SlotState& s = t->slots[slot];
    if (s.elems == 0) return TIDAL_OK;
    if (!s.ready_recorded) return fail(TIDAL_E_STATE, "slot %d was never materialised", slot);
    HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, s.ready, 0));
    return TIDAL_OK;
}

// ---------------------------------------------------------------------------------------
// adapters: validation, packed layout, upload
// ---------------------------------------------------------------------------------------
// keep_rows: also reserve A in row-major form (resident adapters: the unmerged apply contracts
// over the input width and wants A's rows contiguous).
static int validate_targets(const tidal_template* t, const tidal_lora_target* tg, int32_t n, bool need_host,
                            AdapterRec* rec, bool keep_rows = false) {
    if (!t) return fail(TIDAL_E_INVAL, "template is NULL");
    if (n < 0 || (!tg && n > 0)) return fail(TIDAL_E_INVAL, "bad target list (n=%d)", n);
    rec->targets.clear();
    std::vector<char> seen(t->slots.size(), 0);
    size_t off = 0;
    for (int32_t i = 0; i < n; ++i) {
        const tidal_lora_target& g = tg[i];
        if (g.slot < 0 || g.slot >= (int32_t)t->slots.size())
            return fail(TIDAL_E_INVAL, "target %d: slot %d out of range", i, g.slot);
        if (seen[g.slot]) return fail(TIDAL_E_INVAL, "target %d: slot %d given twice", i, g.slot);
        seen[g.slot] = 1;
        if (g.r < 0 || g.r > t->cfg.max_rank)
            return fail(TIDAL_E_INVAL, "target %d: rank %d outside 0..%d", i, g.r, t->cfg.max_rank);
        if (!(g.alpha == g.alpha) || g.alpha - g.alpha != 0.0f)
            return fail(TIDAL_E_INVAL, "target %d: alpha is not finite", i);
        const SlotState& s = t->slots[g.slot];
        if (s.rows > 0x7FFFFFFF || s.cols > 0x7FFFFFFF)
            return fail(TIDAL_E_INVAL, "target %d: slot %d is too large for a LoRA target", i, g.slot);
        PackedTarget p;
        p.slot = g.slot;
        p.r = g.r;
        p.rp = padded_rank(g.r);
        p.alpha = g.alpha;
        p.at_off = p.bp_off = 0;
        p.ar_off = kNoOffset;
        if (p.active() && s.elems > 0) {
            if (!dtype_ok(g.dtype)) return fail(TIDAL_E_INVAL, "target %d: unknown dtype %d", i, g.dtype);
            if (need_host && (!g.A || !g.B)) return fail(TIDAL_E_INVAL, "target %d: A or B is NULL", i);
            // a factor is staged whole: it has to fit one staging buffer
            const size_t longest = (size_t)std::max(s.rows, s.cols) * (size_t)g.r * dtype_size(g.dtype);
            if (need_host && longest > t->cfg.chunk_bytes)
                return fail(TIDAL_E_INVAL, "target %d: a LoRA factor of %zu bytes is larger than chunk_bytes (%zu)", i, longest,
                            t->cfg.chunk_bytes);
            p.at_off = off;
            off = align_up(off + packed_at_bytes(s.cols, p.rp), kSlotAlign);
            p.bp_off = off;
            off = align_up(off + packed_bp_bytes(s.rows, p.rp), kSlotAlign);
            if (keep_rows && s.cols % 8 == 0) {
                p.ar_off = off;
                off = align_up(off + 2 * (size_t)s.cols * p.r, kSlotAlign);
            }
        }
        rec->targets.push_back(p);
    }
    if (off / kLoraUnit > 0xFFFFFFFFull) return fail(TIDAL_E_INVAL, "packed adapter larger than 1 TB");
    rec->bytes = off;
    return TIDAL_OK;
}

static int check_materialised(const tidal_template* t, const AdapterRec& rec) {
    for (const PackedTarget& p : rec.targets)
        if (!t->slots[p.slot].materialised && t->slots[p.slot].elems > 0)
            return fail(TIDAL_E_STATE, "LoRA target slot %d was never materialised", p.slot);
    return TIDAL_OK;
}

extern "C" size_t tidal_adapter_required_bytes(const tidal_template* t, const tidal_lora_target* targets,
                                               int32_t n_targets) {
    AdapterRec rec;
    if (validate_targets(t, targets, n_targets, false, &rec, true)) return 0;
    return rec.bytes ? rec.bytes : kSlotAlign;
}

// Stage A and B of every active target through the staging buffers and pack them into
// rec.dev on `stream`.
// `copy` and `pack` may differ: the copies of a later chunk then run while an earlier one is packed
// (and, for a pipelined attach, merged) on `pack`.  `chunk_io` carries the staging-buffer parity from
// one call to the next so that successive groups alternate between the two buffers.
// A job is one factor staged once; A may be packed twice (transposed and, as a plain conversion
// written as lines of 8, row-major).
struct UploadJob { const char* host; size_t bytes; PackSegment seg; bool pinned; bool has2; PackSegment seg2; };

static int upload_jobs(tidal_template* t, const tidal_lora_target* tg, const AdapterRec& rec, size_t first, size_t last,
                       std::vector<UploadJob>* jobs) {
    for (size_t i = first; i < std::min(last, rec.targets.size()); ++i) {
        const PackedTarget& p = rec.targets[i];
        const SlotState& s = t->slots[p.slot];
        if (!p.active() || s.elems == 0) continue;
        const size_t isz = dtype_size(tg[i].dtype);
        UploadJob a{(const char*)tg[i].A, (size_t)p.r * (size_t)s.cols * isz,
                    PackSegment{nullptr, rec.dev + p.at_off, s.cols, p.r, p.rp, tg[i].dtype, kPackAt}, false, false, {}};
        if (p.ar_off != kNoOffset) {
            a.has2 = true;
            a.seg2 = PackSegment{nullptr, rec.dev + p.ar_off, (int64_t)p.r * s.cols / 8, 8, 8, tg[i].dtype, kPackRows};
        }
        UploadJob b{(const char*)tg[i].B, (size_t)p.r * (size_t)s.rows * isz,
                    PackSegment{nullptr, rec.dev + p.bp_off, s.rows, p.r, p.rp, tg[i].dtype, kPackBp}, false, false, {}};
        if (a.bytes > t->cfg.chunk_bytes || b.bytes > t->cfg.chunk_bytes)
            return fail(TIDAL_E_INVAL, "target %zu: a LoRA factor is larger than chunk_bytes", i);
        jobs->push_back(a);
        jobs->push_back(b);
    }
    for (UploadJob& j : *jobs) j.pinned = host_is_pinned(j.host);
    return TIDAL_OK;
}

static int launch_packs(const std::vector<PackSegment>& segs, hipStream_t stream) {
    for (size_t k = 0; k < segs.size(); k += kMaxPackSeg) {
        const int n = (int)std::min(segs.size() - k, (size_t)kMaxPackSeg);
        PackBatch batch;
        memcpy(batch.seg, segs.data() + k, (size_t)n * sizeof(PackSegment));
        HIP_TRY(launch_pack(batch, n, stream));
    }
    return TIDAL_OK;
}

// Stage the factors of an adapter chunk by chunk through the two staging buffers and pack them into
// rec.dev: copies on `copy`, pack kernels on `pack` (the same stream or two).
static int upload_adapter(tidal_template* t, const tidal_lora_target* tg, const AdapterRec& rec, hipStream_t copy,
                          hipStream_t pack) {
    typedef UploadJob Job;
    std::vector<Job> jobs;
    int rc0 = upload_jobs(t, tg, rec, 0, rec.targets.size(), &jobs);
    if (rc0) return rc0;
    if (jobs.empty()) return TIDAL_OK;

    Pipeline pl{t, copy, pack};
    pl.kernel_copy = true;
    size_t i = 0;
    int chunk = 0;
    while (i < jobs.size()) {
        const int b = chunk & 1;
        // fill one staging buffer with whole factors: all copies first (neighbouring ones merge
        // into one DMA), then the pack launches, so that a chunk pays the copy -> kernel hand-over once
        size_t fill = 0, j = i;
        bool need_bounce = false;
        std::vector<size_t> offs;
        while (j < jobs.size()) {
            size_t off = align_up(fill, kSlotAlign);
            if (off + jobs[j].bytes > t->cfg.chunk_bytes) break;
            offs.push_back(off);
            fill = off + jobs[j].bytes;
            need_bounce |= !jobs[j].pinned || jobs[j].bytes < t->cfg.coalesce_bytes;
            ++j;
        }
        int rc = pl.acquire(b, need_bounce, true);
        if (rc) return rc;
        std::vector<PackSegment> segs;
        for (size_t k = i; k < j; ++k) {
            Job& job = jobs[k];
            const bool gathered = !job.pinned || job.bytes < t->cfg.coalesce_bytes;
            char* dst = t->arena + t->lay.staging[b] + offs[k - i];
            rc = pl.put(gathered, b, (int64_t)offs[k - i], job.host, job.bytes, dst);
            if (rc) return rc;
            job.seg.src = dst;
            segs.push_back(job.seg);
            if (job.has2) {
                job.seg2.src = dst;
                segs.push_back(job.seg2);
            }
        }
        rc = pl.copies_done(b, need_bounce, true);
        if (rc) return rc;
        rc = launch_packs(segs, pack);
        if (rc) return rc;
        rc = pl.consumed(b);
        if (rc) return rc;
        i = j;
        ++chunk;
    }
    return TIDAL_OK;
}

extern "C" int tidal_adapter_upload(tidal_template* t, const tidal_lora_target* targets, int32_t n_targets,
                                    void* dev_mem, size_t dev_bytes, void* stream, tidal_adapter** out) {
    if (!out) return fail(TIDAL_E_INVAL, "out is NULL");
    *out = nullptr;
    AdapterRec rec;
    int rc = validate_targets(t, targets, n_targets, true, &rec, true);
    if (rc) return rc;
    if (!dev_mem) return fail(TIDAL_E_INVAL, "dev_mem is NULL");
    if ((uintptr_t)dev_mem % kSlotAlign) return fail(TIDAL_E_INVAL, "dev_mem is not 256-byte aligned");
    if (rec.bytes > dev_bytes) return fail(TIDAL_E_NOMEM, "adapter needs %zu bytes, got %zu", rec.bytes, dev_bytes);
    rc = ensure_device(t);
    if (rc) return rc;
    rec.dev = (char*)dev_mem;
    tidal_adapter* a = new (std::nothrow) tidal_adapter();
    if (!a) return fail(TIDAL_E_NOMEM, "out of host memory");
    hipError_t e = hipEventCreateWithFlags(&rec.ready, hipEventDisableTiming);
    if (e != hipSuccess) {
        delete a;
        return fail(TIDAL_E_HIP, "hipEventCreate failed: %s", hipGetErrorString(e));
    }
    // the staging buffers are shared with materialisations and other uploads, whatever their streams
    rc = wait_marks(t, kMarkLoad, (hipStream_t)stream);
    if (!rc) rc = upload_adapter(t, targets, rec, (hipStream_t)stream, (hipStream_t)stream);
    if (!rc && hipEventRecord(rec.ready, (hipStream_t)stream) != hipSuccess) rc = fail(TIDAL_E_HIP, "hipEventRecord failed");
    if (!rc) rc = mark_done(t, kMarkLora, (hipStream_t)stream);
    if (rc) {
        (void)hipStreamSynchronize((hipStream_t)stream);       // nothing may still read the caller's host memory
        (void)hipEventDestroy(rec.ready);
        delete a;
        return rc;
    }
    a->owner = t;
    a->rec = rec;
    a->attached = false;
    *out = a;
    return TIDAL_OK;
}

extern "C" int tidal_adapter_destroy(tidal_adapter* a) {
    if (!a) return TIDAL_OK;
    if (a->attached) return fail(TIDAL_E_STATE, "adapter is attached; detach or swap it out first");
    if (a->rec.ready) (void)hipEventDestroy(a->rec.ready);
    delete a;
    return TIDAL_OK;
}

// ---------------------------------------------------------------------------------------
// LoRA launches
// ---------------------------------------------------------------------------------------
typedef std::tuple<int64_t, int64_t, int, int, int, int> LoraKey;   // out, in, rp_old, rp_new, r_old, r_new

// One launch per (shape, ranks) group and at most kMaxLoraTargets slots; a larger group is cut
// into equal parts (160 slots: 80 + 80, not 128 + 32 -- the short launch would run at a lower rate).
static int launch_groups(tidal_template* t, const std::map<LoraKey, std::vector<LoraTargetDev>>& groups,
                         const char* old_base, const char* new_base, bool fork, hipStream_t stream) {
    const bool ordered = (t->cfg.flags & TIDAL_FLAG_ORDERED_ACCUM) != 0;
    for (auto& g : groups) {
        const std::vector<LoraTargetDev>& all = g.second;
        const size_t parts = (all.size() + kMaxLoraTargets - 1) / kMaxLoraTargets;
        const size_t per = parts ? (all.size() + parts - 1) / parts : 0;
        for (size_t at = 0; at < all.size(); at += per) {
            const size_t n = std::min(all.size() - at, per);
            LoraBatch batch;
            batch.w_base = t->arena;
            batch.old_base = old_base;
            batch.new_base = new_base;
            memcpy(batch.t, all.data() + at, n * sizeof(LoraTargetDev));
            LoraGroup lg;
            lg.batch = &batch;
            lg.n_targets = (int32_t)n;
            lg.out = (int32_t)std::get<0>(g.first);
            lg.in = (int32_t)std::get<1>(g.first);
            lg.rp_old = std::get<2>(g.first);
            lg.rp_new = std::get<3>(g.first);
            lg.r_old = std::get<4>(g.first);
            lg.r_new = std::get<5>(g.first);
            lg.fork = fork;
            const LoraLaunchPlan plan = plan_lora_launch(lg, ordered);
            if (plan.kind == kLoraNone) continue;
            hipEvent_t t0;
            int trc = timing_begin(t, stream, &t0);
            if (trc) return trc;
            HIP_TRY(ordered ? launch_lora_ordered(lg, stream) : launch_lora_mfma(lg, plan, stream));
            trc = timing_end(t, stream, t0, true);
            if (trc) return trc;
            t->stats.lora_launches++;
        }
    }
    return TIDAL_OK;
}

// Which kernel, variant, walk length and grid a LoRA pass over n_targets slots of out x in would
// be launched with (host-only introspection, like tidal_materialize_plan).
extern "C" int tidal_lora_launch_info(const tidal_template* t, int64_t out, int64_t in, int32_t n_targets,
                                      int32_t r_old, int32_t r_new, int32_t fork, tidal_lora_launch* info) {
    if (!t || !info) return fail(TIDAL_E_INVAL, "NULL argument");
    if (out <= 0 || in <= 0 || out > 0x7FFFFFFF || in > 0x7FFFFFFF) return fail(TIDAL_E_INVAL, "bad shape");
    if (n_targets <= 0) return fail(TIDAL_E_INVAL, "n_targets must be positive");
    if (r_old < 0 || r_new < 0 || r_old > t->cfg.max_rank || r_new > t->cfg.max_rank)
        return fail(TIDAL_E_INVAL, "rank outside 0..%d", t->cfg.max_rank);
    if (fork && r_old) return fail(TIDAL_E_INVAL, "a fork apply has no old adapter");
    memset(info, 0, sizeof *info);
    const size_t parts = ((size_t)n_targets + kMaxLoraTargets - 1) / kMaxLoraTargets;
    const size_t per = ((size_t)n_targets + parts - 1) / parts;
    LoraGroup lg;
    lg.batch = nullptr;
    lg.n_targets = (int32_t)per;
    lg.out = (int32_t)out;
    lg.in = (int32_t)in;
    lg.r_old = r_old;
    lg.r_new = r_new;
    lg.rp_old = padded_rank(r_old);
    lg.rp_new = padded_rank(r_new);
    lg.fork = fork != 0;
    const LoraLaunchPlan p = plan_lora_launch(lg, (t->cfg.flags & TIDAL_FLAG_ORDERED_ACCUM) != 0);
    info->launches = p.kind == kLoraNone ? 0 : (int32_t)parts;
    info->targets_per_launch = (int32_t)per;
    info->rank_padded_old = 16 * p.ks_old;
    info->rank_padded_new = 16 * p.ks_new;
    info->blocks_per_walk = p.rc;
    info->waves_per_simd = p.waves_per_simd;
    info->workgroups = p.total_blocks;
    switch (p.kind) {
        case kLoraMfmaReg:
            snprintf(info->kernel, sizeof info->kernel, "lora_mfma_kernel<8,%d,%d,%s,%s>", p.ks_old, p.ks_new,
                     p.fork ? "fork" : "inplace", p.pair ? "pair" : "all");
            break;
        case kLoraMfmaLds:
            snprintf(info->kernel, sizeof info->kernel, "lora_mfma_lds_kernel<8,%d,%d>", p.ks_old, p.ks_new);
            break;
        case kLoraOrdered: snprintf(info->kernel, sizeof info->kernel, "lora_ordered_kernel"); break;
        default: snprintf(info->kernel, sizeof info->kernel, "none"); break;
    }
    return TIDAL_OK;
}

// One pass over the union of the slots of `older` (subtracted) and `newer` (added); either
// may be NULL.  Slots are grouped by (shape, padded ranks) and each group is one launch.
static int launch_rmw(tidal_template* t, const AdapterRec* older, const AdapterRec* newer, hipStream_t stream) {
    struct Side { const PackedTarget* p; const AdapterRec* rec; };
    std::map<int32_t, std::pair<Side, Side>> by_slot;
    if (older)
        for (const PackedTarget& p : older->targets)
            if (p.active() && t->slots[p.slot].elems > 0) by_slot[p.slot].first = Side{&p, older};
    if (newer)
        for (const PackedTarget& p : newer->targets)
            if (p.active() && t->slots[p.slot].elems > 0) by_slot[p.slot].second = Side{&p, newer};
    if (by_slot.empty()) return TIDAL_OK;
    // the slots may still be streaming in on the materialisation's streams, and a resident adapter
    // may still be uploading on the stream it was given
    int wrc = wait_marks(t, kMarkLoad, stream);
    if (wrc) return wrc;
    if (older && older->ready) HIP_TRY(hipStreamWaitEvent(stream, older->ready, 0));
    if (newer && newer->ready) HIP_TRY(hipStreamWaitEvent(stream, newer->ready, 0));

    typedef LoraKey Key;
    std::map<Key, std::vector<LoraTargetDev>> groups;
    for (auto& kv : by_slot) {
        const SlotState& s = t->slots[kv.first];
        const Side& o = kv.second.first;
        const Side& n = kv.second.second;
        LoraTargetDev d;
        memset(&d, 0, sizeof d);
        if (t->lay.slot_offset[kv.first] / kLoraUnit > 0xFFFFFFFFull)      // descriptors hold 32-bit offsets in 256-byte units
            return fail(TIDAL_E_INVAL, "slot %d lies beyond 1 TB from the start of the arena", kv.first);
        d.w = (uint32_t)(t->lay.slot_offset[kv.first] / kLoraUnit);
        int rp_old = 0, rp_new = 0, r_old = 0, r_new = 0;
        if (o.p) {
            d.at_old = (uint32_t)(o.p->at_off / kLoraUnit);
            d.bp_old = (uint32_t)(o.p->bp_off / kLoraUnit);
            d.s_old = -(o.p->alpha / (float)o.p->r);
            rp_old = o.p->rp;
            r_old = o.p->r;
        }
        if (n.p) {
            d.at_new = (uint32_t)(n.p->at_off / kLoraUnit);
            d.bp_new = (uint32_t)(n.p->bp_off / kLoraUnit);
            d.s_new = n.p->alpha / (float)n.p->r;
            rp_new = n.p->rp;
            r_new = n.p->r;
        }
        groups[Key(s.rows, s.cols, rp_old, rp_new, r_old, r_new)].push_back(d);
        t->stats.rmw_elems += (uint64_t)s.elems;
    }
    int rc = launch_groups(t, groups, older ? older->dev : nullptr, newer ? newer->dev : nullptr, false, stream);
    if (rc) return rc;
    return mark_done(t, kMarkLora, stream);
}

static int do_swap_launch(tidal_template* t, const AdapterRec* older, const AdapterRec* newer, hipStream_t stream) {
    if ((t->cfg.flags & TIDAL_FLAG_TWO_PASS_SWAP) && older && newer) {
        int rc = launch_rmw(t, older, nullptr, stream);
        if (rc) return rc;
        return launch_rmw(t, nullptr, newer, stream);
    }
    return launch_rmw(t, older, newer, stream);
}

static void set_attached(tidal_template* t, const AdapterRec& rec, tidal_adapter* resident, int region) {
    if (t->cur_resident) t->cur_resident->attached = false;
    t->attached = true;
    t->cur = rec;
    t->cur_resident = resident;
    t->cur_region = region;
    if (resident) resident->attached = true;
}

// Rates the grouping of a pipelined attach is sized from.  They start at typical values and are
// replaced by what the library measures with its own events on a pipelined call: the link rate from
// the first group's copies (alone on their stream), the in-place pass rate from the last group's launches.
static void rates_update(tidal_template* t) {
    RateModel& r = t->rates;
    if (!r.pending) return;
    if (hipEventQuery(r.ev[1]) != hipSuccess || hipEventQuery(r.ev[3]) != hipSuccess) {
        (void)hipGetLastError();           // still running: keep the current estimates
        return;
    }
    float up_ms = 0.f, rmw_ms = 0.f;
    // copies of a few megabytes and more run at the link's rate; smaller ones measure latency: keep the estimate then
    // (and a copy that shared the link or waited for its turn reads low: the estimate only drifts down slowly)
    if (hipEventElapsedTime(&up_ms, r.ev[0], r.ev[1]) == hipSuccess && up_ms > 1e-3f && r.up_bytes >= 8.0e6)
        r.link_bytes_per_ms = std::max(0.9 * r.link_bytes_per_ms, r.up_bytes / up_ms);
    if (hipEventElapsedTime(&rmw_ms, r.ev[2], r.ev[3]) == hipSuccess && rmw_ms > 1e-3f && r.rmw_bytes > 0.0)
        r.rmw_bytes_per_ms = r.rmw_bytes / rmw_ms;
    (void)hipGetLastError();
    r.pending = false;
}

// The two staging buffers lie back to back in the arena: one span for the grouped upload.
static inline size_t staging_span(const tidal_template* t) { return 2 * t->cfg.chunk_bytes; }

// Cut the targets of an adapter given by host pointers into groups that are uploaded and merged in
// turn.  With upload time u and merge time m of each target known from the two rates, the end of
// the call is simulated for every choice of the first group's size (each later group: as many
// targets as cross the link while the group before it is merged) and the best one taken.  Every
// launch is charged a fixed cost, which keeps the number of groups down; small adapters, one
// target, or TIDAL_FLAG_SERIAL_UPLOAD give a single group (one stream, no pipelining).
static void plan_upload_groups(const tidal_template* t, const tidal_lora_target* tg, const AdapterRec& rec,
                               const AdapterRec* old, std::vector<std::pair<size_t, size_t>>* groups) {
    constexpr size_t kPipelineFrom = (size_t)4 << 20;
    constexpr double kLaunchMs = 0.02;             // what one more launch costs: its bubble, its ramp and tail
    constexpr double kWaitMs = 0.04;               // what a cross-stream wait costs the calling thread
    constexpr double kHandoverMs = 0.03;           // from the end of a group's copies to the start of its pack on the other stream
    constexpr double kGroupMs = 0.035;             // what one more group costs the caller's stream (measured on 64 targets of 4096 x 4096)
    const size_t n = rec.targets.size();
    groups->clear();
    groups->push_back({0, n});
    const bool forced = (t->cfg.flags & TIDAL_FLAG_PIPELINED_UPLOAD) != 0;
    if ((t->cfg.flags & TIDAL_FLAG_SERIAL_UPLOAD) || n < 2 || (!forced && rec.bytes < kPipelineFrom)) return;
    std::vector<char> in_old(t->slots.size(), 0);
    if (old)
        for (const PackedTarget& p : old->targets)
            if (p.active()) in_old[p.slot] = 1;
    std::vector<double> u(n, 0.0), m(n, 0.0), raw(n, 0.0);
    double u_total = 0.0, m_total = 0.0;
    for (size_t i = 0; i < n; ++i) {
        const PackedTarget& p = rec.targets[i];
        const SlotState& s = t->slots[p.slot];
        if (s.elems == 0) continue;
        if (p.active()) raw[i] = (double)p.r * (double)(s.rows + s.cols) * (double)dtype_size(tg[i].dtype) + 2.0 * kSlotAlign;
        u[i] = raw[i] / t->rates.link_bytes_per_ms;
        if (p.active() || in_old[p.slot]) m[i] = 4.0 * (double)s.elems / t->rates.rmw_bytes_per_ms;
        u_total += u[i];
        m_total += m[i];
    }
    if (u_total <= 0.0 || m_total <= 0.0) return;
    // shape classes of a range of targets = launches of its merge
    auto launches = [&](size_t a, size_t b) {
        int cnt = 0;
        int64_t seen[8][2];
        for (size_t i = a; i < b && cnt < 8; ++i) {
            const SlotState& s = t->slots[rec.targets[i].slot];
            bool found = false;
            for (int k = 0; k < cnt; ++k) found |= seen[k][0] == s.rows && seen[k][1] == s.cols;
            if (!found) { seen[cnt][0] = s.rows; seen[cnt][1] = s.cols; ++cnt; }
        }
        return cnt < 1 ? 1 : cnt;
    };
    // a single group (serial) is the candidate to beat, unless grouping is forced
    double best = forced ? 1e300 : u_total + m_total + kLaunchMs * launches(0, n);
    std::vector<std::pair<size_t, size_t>> best_groups = *groups;
    // Candidates: G groups whose shares of the upload grow by a factor q from one to the next
    // (q = 1: equal groups, what an upload-bound adapter wants; q > 1: a small first group, so that
    // merging starts early, and large later ones that hide under the merges before them).  Each is
    // simulated on three resources -- the link, the packing stream, the caller's stream -- and the
    // one that ends first is taken.
    const double pack_rate = 2.0e9;                                      // bytes per ms through the pack kernel
    static const double kGrowth[] = {1.0, 1.5, 2.0, 3.0};
    static const double kFirst[] = {1.0, 0.35};                           // the first group may be smaller still
    for (int G = 2; G <= kMaxUploadGroups && (size_t)G <= n; ++G) {
        for (int v = 0; v < 8; ++v) {
            const double q = kGrowth[v & 3], f0 = kFirst[v >> 2];
            double norm = 0.0, w = 1.0;
            for (int g = 0; g < G; ++g) { norm += g ? w : f0; w *= q; }
            std::vector<std::pair<size_t, size_t>> cand;
            size_t a0 = 0;
            double share = 0.0, acc = 0.0;
            w = 1.0;
            for (int g = 0; g < G; ++g) {
                share += (g ? w : f0) / norm;
                w *= q;
                size_t b0 = a0;
                while (b0 < n && (acc + u[b0] <= share * u_total + 1e-12 || b0 == a0)) acc += u[b0++];
                if (g == G - 1) b0 = n;
                if (b0 > a0) cand.push_back({a0, b0});
                a0 = b0;
                if (a0 >= n) break;
            }
            if (cand.size() < 2) continue;
            // the link carries the groups back to back, as soon as the calling thread has got to them; the
            // caller's stream takes each group when its copies are in: pack, then merge
            // (the first group's copies run on the caller's stream and share the link with the second's)
            double link_done = kWaitMs, merge_done = 0.0;
            bool fits = true, first_group = true;
            for (const auto& gr : cand) {
                double ug = 0.0, mg = 0.0, bytes = 0.0;
                for (size_t i = gr.first; i < gr.second; ++i) { ug += u[i]; mg += m[i]; bytes += raw[i]; }
                fits = fits && bytes <= 0.5 * (double)staging_span(t);
                link_done += ug;                                 // the link's total does not depend on who shares it
                const double here = first_group ? 1.5 * ug : link_done + kHandoverMs;
                merge_done = std::max(merge_done, here) + 2.0 * bytes / pack_rate + mg + kGroupMs +
                             kLaunchMs * (launches(gr.first, gr.second) - 1);
                first_group = false;
            }
            if (!fits) continue;
            if (merge_done < best) {
                best = merge_done;
                best_groups = cand;
            }
        }
    }
    *groups = best_groups;
    const TuningKnobs knobs = tuning_knobs();                 // tuning builds only: targets per group, given outright
    if (knobs.n_up_groups > 0) {
        std::vector<std::pair<size_t, size_t>> forced_groups;
        size_t a0 = 0;
        for (int k = 0; k < knobs.n_up_groups && a0 < n; ++k) {
            forced_groups.push_back({a0, std::min(n, a0 + (size_t)knobs.up_groups[k])});
            a0 = forced_groups.back().second;
        }
        if (a0 < n) forced_groups.push_back({a0, n});
        if (forced_groups.size() <= (size_t)kMaxUploadGroups) *groups = forced_groups;
    }
    if (host_trace_on()) {
        fprintf(stderr, "[groups]");
        for (const auto& gr : *groups) fprintf(stderr, " %zu", gr.second - gr.first);
        fprintf(stderr, "  (link %.1f GB/s, pass %.2f TB/s)\n", t->rates.link_bytes_per_ms / 1e6, t->rates.rmw_bytes_per_ms / 1e9);
    }
}

// attach (swap = false) or swap (swap = true) an adapter given by host pointers
static int attach_host(tidal_template* t, const tidal_lora_target* tg, int32_t n, void* stream, bool swap) {
    AdapterRec rec;
    int rc = validate_targets(t, tg, n, true, &rec);
    if (rc) return rc;
    if (!swap && t->attached) return fail(TIDAL_E_STATE, "an adapter is already attached");
    if (swap && !t->attached) return fail(TIDAL_E_STATE, "no adapter is attached");
    rc = check_materialised(t, rec);
    if (rc) return rc;
    if (rec.bytes > t->cfg.max_adapter_bytes)
        return fail(TIDAL_E_NOMEM, "packed adapter needs %zu bytes, max_adapter_bytes is %zu", rec.bytes,
                    t->cfg.max_adapter_bytes);
    rc = ensure_device(t);
    if (rc) return rc;
    const int region = (t->cur_region == 0) ? 1 : 0;
    rec.dev = t->arena + t->lay.adapter_region[region];
    AdapterRec old = t->cur;

    // Upload and merge in groups of targets: while group g is packed and merged on the caller's
    // stream, the copies of group g+1 cross the link on a stream of the library's own.
    std::vector<std::pair<size_t, size_t>> groups;
    plan_upload_groups(t, tg, rec, swap ? &old : nullptr, &groups);
    // the grouped path copies straight from the caller's memory: pinned factors only, each group's share
    // of the staging memory in one piece
    std::vector<std::vector<UploadJob>> group_jobs;
    if (groups.size() > 1) {
        bool ok = true;
        for (const auto& gr : groups) {
            group_jobs.emplace_back();
            rc = upload_jobs(t, tg, rec, gr.first, gr.second, &group_jobs.back());
            if (rc) return rc;
            size_t need = 0;
            for (const UploadJob& j : group_jobs.back()) {
                need = align_up(need, kSlotAlign) + j.bytes;
                ok = ok && j.pinned;
            }
            ok = ok && need <= staging_span(t);
        }
        if (!ok) groups.assign(1, {0, rec.targets.size()});
    }
    if (groups.size() <= 1) {
        rc = upload_adapter(t, tg, rec, (hipStream_t)stream, (hipStream_t)stream);
        if (rc) return rc;
        rc = do_swap_launch(t, swap ? &old : nullptr, &rec, (hipStream_t)stream);
        if (rc) return rc;
    } else {
        rc = ensure_upload_stream(t);
        if (rc) return rc;
        rates_update(t);
        // Two streams, and as few cross-stream waits as possible (each costs the calling thread tens of
        // microseconds, more than a launch).  The first group stays on the caller's stream altogether:
        // copy, pack, merge, no event.  The copies of all later groups go to the library's stream at once,
        // back to back from the start, each group into its own piece of the staging memory; the caller's
        // stream waits once per group for that group's copies, packs it and merges it.
        hipStream_t cs = (hipStream_t)stream;
        const size_t G = groups.size();
        rc = wait_marks(t, kMarkLora, cs);                       // the region may still be read by a pass on another stream
        if (rc) return rc;
        HIP_TRY(hipEventRecord(t->ev_up_begin, cs));             // staging memory: last used on the caller's stream ...
        HIP_TRY(hipStreamWaitEvent(t->up_stream, t->ev_up_begin, 0));
        for (int b = 0; b < 2; ++b)                              // ... or on some other one
            if (t->staging_rec[b] && t->staging_stream[b] != cs) {
                HIP_TRY(hipStreamWaitEvent(t->up_stream, t->staging_free[b], 0));
                HIP_TRY(hipStreamWaitEvent(cs, t->staging_free[b], 0));
            }
        const bool calibrate = !t->rates.pending;
        std::vector<char> in_new(t->slots.size(), 0);
        for (const PackedTarget& p : rec.targets) in_new[p.slot] = 1;
        const size_t cap = staging_span(t);
        struct Span { size_t lo, hi; };
        std::vector<Span> spans;                                 // staging bytes of the groups whose copies are enqueued
        std::vector<std::vector<PackSegment>> group_segs(G);
        size_t pos = 0;
        HostTrace trace;                                         // tuning builds: host time of each step; nothing otherwise
        auto hmark = [&](const char* what, size_t g) { trace.mark(what, g); };
        // Enqueue the copies of the next groups, as far as their pieces of staging memory are free or
        // become free behind packs that are enqueued already (those of groups < packed_upto).
        size_t copied_upto = 0;
        auto enqueue_copies = [&](size_t packed_upto) -> int {
            while (copied_upto < G) {
                const size_t g = copied_upto;
                hipStream_t on = g == 0 ? cs : t->up_stream;
                const auto& jobs = group_jobs[g];
                size_t need = 0;
                for (const UploadJob& j : jobs) need = align_up(need, kSlotAlign) + j.bytes;
                size_t at = pos + need > cap ? 0 : pos;          // groups never straddle the end (each fits: checked above)
                for (size_t k = 0; k < spans.size(); ++k)
                    if (spans[k].lo < at + need && at < spans[k].hi && k >= packed_upto) return TIDAL_OK;   // not yet
                for (size_t k = 0; k < spans.size(); ++k)
                    if (spans[k].lo < at + need && at < spans[k].hi) {
                        HIP_TRY(hipStreamWaitEvent(on, t->ev_group_packed[k], 0));
                        spans[k].lo = spans[k].hi = 0;
                    }
                const bool timed = calibrate && g + 1 == G;      // the last group has the link to itself
                if (timed) HIP_TRY(hipEventRecord(t->rates.ev[0], on));
                Pipeline pl{t, on, on};
                pl.kernel_copy = true;
                // the first group's pack follows on the same stream: a kernel that fetches the factors spares the
                // hand-over from the copy engine, which costs more than a few megabytes take to cross the link
                if (g == 0) pl.kernel_copy_max = (size_t)8 << 20;
                size_t off = at;
                double up_bytes = 0.0;
                for (const UploadJob& job : jobs) {
                    off = align_up(off, kSlotAlign);
                    char* dst = t->arena + t->lay.staging[0] + off;
                    int prc = pl.put(false, 0, 0, job.host, job.bytes, dst);
                    if (prc) return prc;
                    PackSegment sg = job.seg;
                    sg.src = dst;
                    group_segs[g].push_back(sg);
                    if (job.has2) {
                        sg = job.seg2;
                        sg.src = dst;
                        group_segs[g].push_back(sg);
                    }
                    off += job.bytes;
                    up_bytes += (double)job.bytes;
                }
                int prc = pl.flush();
                if (!prc) prc = pl.flush_kernel_copies();
                if (prc) return prc;
                spans.push_back(Span{at, at + need});
                pos = at + need;
                if (timed) {
                    HIP_TRY(hipEventRecord(t->rates.ev[1], on));
                    t->rates.up_bytes = up_bytes;
                }
                if (g > 0) HIP_TRY(hipEventRecord(t->ev_group_copied[g], on));
                hmark("copies", g);
                ++copied_upto;
            }
            return TIDAL_OK;
        };
        for (size_t g = 0; g < G; ++g) {
            rc = enqueue_copies(g);                              // at least group g's, as a rule all that are left
            if (rc) return rc;
            if (copied_upto <= g) return fail(TIDAL_E_STATE, "internal: group %zu has no staging memory", g);
            if (g > 0) HIP_TRY(hipStreamWaitEvent(cs, t->ev_group_copied[g], 0));
            rc = launch_packs(group_segs[g], cs);
            if (rc) return rc;
            if (g + 1 < G) HIP_TRY(hipEventRecord(t->ev_group_packed[g], cs));   // a later group may want this piece
            AdapterRec part_new, part_old;
            part_new.dev = rec.dev;
            part_new.targets.assign(rec.targets.begin() + groups[g].first, rec.targets.begin() + groups[g].second);
            if (swap) {
                std::vector<char> here(t->slots.size(), 0);
                for (const PackedTarget& p : part_new.targets) here[p.slot] = 1;
                part_old.dev = old.dev;
                for (const PackedTarget& p : old.targets)       // slots only the old adapter touches go last
                    if (here[p.slot] || (g + 1 == G && !in_new[p.slot])) part_old.targets.push_back(p);
            }
            const bool last = g + 1 == G;
            if (last) {
                // later users of the staging buffers, on whatever stream, order themselves behind the packs
                for (int b = 0; b < 2; ++b) {
                    HIP_TRY(hipEventRecord(t->staging_free[b], cs));
                    t->staging_rec[b] = true;
                    t->staging_stream[b] = cs;
                }
            }
            if (last && calibrate) HIP_TRY(hipEventRecord(t->rates.ev[2], cs));
            const uint64_t before = t->stats.rmw_elems;
            rc = do_swap_launch(t, swap ? &part_old : nullptr, &part_new, cs);
            if (rc) return rc;
            hmark("launched", g);
            if (last && calibrate) {
                HIP_TRY(hipEventRecord(t->rates.ev[3], cs));
                t->rates.rmw_bytes = 4.0 * (double)(t->stats.rmw_elems - before);
                t->rates.pending = true;
            }
        }
    }
    host_call_report();
    set_attached(t, rec, nullptr, region);
    return TIDAL_OK;
}

extern "C" int tidal_materialize_attach(tidal_template* t, const tidal_src* srcs, int32_t n_src,
                                        const tidal_lora_target* targets, int32_t n_targets, void* copy_stream,
                                        void* compute_stream) {
    std::vector<SourceInfo> infos;
    int rc = gather_sources(t, srcs, n_src, 0, &infos);
    if (rc) return rc;
    AdapterRec rec;
    rc = validate_targets(t, targets, n_targets, true, &rec);
    if (rc) return rc;
    bool clears = false;
    rc = check_rematerialise(t, infos, &clears);
    if (rc) return rc;
    if (t->attached && !clears)
        return fail(TIDAL_E_STATE, "an adapter is attached and this call does not re-materialise its slots");
    std::vector<char> covered(t->slots.size(), 0);
    for (const SourceInfo& s : infos) covered[s.slot] = 1;
    for (const PackedTarget& p : rec.targets)
        if (p.active() && t->slots[p.slot].elems > 0 && !covered[p.slot])
            return fail(TIDAL_E_INVAL, "LoRA target slot %d is not among the sources", p.slot);
    if (rec.bytes > t->cfg.max_adapter_bytes)
        return fail(TIDAL_E_NOMEM, "packed adapter needs %zu bytes, max_adapter_bytes is %zu", rec.bytes,
                    t->cfg.max_adapter_bytes);
    rc = ensure_device(t);
    if (rc) return rc;
    const int region = (t->cur_region == 0) ? 1 : 0;
    rec.dev = t->arena + t->lay.adapter_region[region];
    // the factors go first, on the compute stream, where the kernels that read them run
    rc = wait_marks(t, kMarkLora, (hipStream_t)compute_stream);
    if (rc) return rc;
    rc = wait_marks(t, kMarkLoad, (hipStream_t)compute_stream);
    if (rc) return rc;
    rc = upload_adapter(t, targets, rec, (hipStream_t)compute_stream, (hipStream_t)compute_stream);
    if (rc) return rc;
    rc = materialize_impl(t, infos, clears, copy_stream, compute_stream, &rec);
    if (rc) return rc;
    set_attached(t, rec, nullptr, region);
    return TIDAL_OK;
}

extern "C" int tidal_lora_attach(tidal_template* t, const tidal_lora_target* targets, int32_t n_targets, void* stream) {
    return attach_host(t, targets, n_targets, stream, false);
}

extern "C" int tidal_lora_swap(tidal_template* t, const tidal_lora_target* targets_new, int32_t n_targets, void* stream) {
    return attach_host(t, targets_new, n_targets, stream, true);
}

static int attach_resident(tidal_template* t, const tidal_adapter* a_c, void* stream, bool swap) {
    if (!t || !a_c) return fail(TIDAL_E_INVAL, "NULL argument");
    tidal_adapter* a = const_cast<tidal_adapter*>(a_c);
    if (a->owner != t) return fail(TIDAL_E_INVAL, "adapter belongs to another template");
    if (!swap && t->attached) return fail(TIDAL_E_STATE, "an adapter is already attached");
    if (swap && !t->attached) return fail(TIDAL_E_STATE, "no adapter is attached");
    int rc = check_materialised(t, a->rec);
    if (rc) return rc;
    rc = ensure_device(t);
    if (rc) return rc;
    AdapterRec old = t->cur;
    rc = do_swap_launch(t, swap ? &old : nullptr, &a->rec, (hipStream_t)stream);
    if (rc) return rc;
    set_attached(t, a->rec, a, -1);
    return TIDAL_OK;
}

extern "C" int tidal_lora_attach_adapter(tidal_template* t, const tidal_adapter* a, void* stream) {
    return attach_resident(t, a, stream, false);
}

extern "C" int tidal_lora_swap_adapter(tidal_template* t, const tidal_adapter* a_new, void* stream) {
    return attach_resident(t, a_new, stream, true);
}

// ---------------------------------------------------------------------------------------
// unmerged adapters applied to a mixed batch
// ---------------------------------------------------------------------------------------
extern "C" size_t tidal_lora_apply_workspace_bytes(int32_t n_tokens) {
    if (n_tokens <= 0) return kSlotAlign;
    return align_up((size_t)n_tokens * kApplyRankStride * 2, kSlotAlign);
}

static int lora_apply_impl(tidal_template* t, const int32_t* slots, int32_t n_slots,
                           const tidal_adapter* const* adapters, int32_t n_adapters, const tidal_lora_segment* segs,
                           int32_t n_segs, const void* x, void* const* ys, int32_t n_tokens, void* workspace,
                           size_t workspace_bytes, void* stream_, bool no_alloc = false) {
    if (!t) return fail(TIDAL_E_INVAL, "template is NULL");
    if (n_slots < 0 || (!slots && n_slots > 0)) return fail(TIDAL_E_INVAL, "bad slot list");
    if (n_adapters < 0 || (!adapters && n_adapters > 0)) return fail(TIDAL_E_INVAL, "bad adapter list");
    if (n_segs < 0 || (!segs && n_segs > 0)) return fail(TIDAL_E_INVAL, "bad segment list");
    if (n_tokens < 0) return fail(TIDAL_E_INVAL, "n_tokens is negative");
    int64_t in = -1;
    for (int32_t k = 0; k < n_slots; ++k) {
        const int32_t slot = slots[k];
        if (slot < 0 || slot >= (int32_t)t->slots.size()) return fail(TIDAL_E_INVAL, "slot %d out of range", slot);
        for (int32_t m = 0; m < k; ++m)
            if (slots[m] == slot) return fail(TIDAL_E_INVAL, "slot %d given twice", slot);
        const SlotState& st = t->slots[slot];
        if (st.rows > 0x7FFFFFFF || st.cols > 0x7FFFFFFF) return fail(TIDAL_E_INVAL, "slot %d is too large", slot);
        if (st.elems > 0 && (st.cols % 8 || st.rows % 8))
            return fail(TIDAL_E_INVAL, "slot %d is %lld x %lld: both must be multiples of 8", slot, (long long)st.rows,
                        (long long)st.cols);
        if (in >= 0 && st.cols != in)
            return fail(TIDAL_E_INVAL, "slot %d has %lld input columns, slot %d has %lld: the targets of one call share x",
                        slot, (long long)st.cols, slots[0], (long long)in);
        in = st.cols;
    }
    // per (adapter, slot): the adapter's entry for that slot
    std::vector<const PackedTarget*> entry((size_t)n_adapters * (size_t)std::max(n_slots, 1), nullptr);
    for (int32_t a = 0; a < n_adapters; ++a) {
        if (!adapters[a]) return fail(TIDAL_E_INVAL, "adapter %d is NULL", a);
        if (adapters[a]->owner != t) return fail(TIDAL_E_INVAL, "adapter %d belongs to another template", a);
        const tidal_adapter* ad = adapters[a];
        if (ad->target_of_slot.empty()) {
            ad->target_of_slot.assign(t->slots.size(), -1);
            for (size_t i = 0; i < ad->rec.targets.size(); ++i) ad->target_of_slot[ad->rec.targets[i].slot] = (int32_t)i;
        }
        for (int32_t k = 0; k < n_slots; ++k) {
            const int32_t at = ad->target_of_slot[slots[k]];
            if (at < 0) return fail(TIDAL_E_INVAL, "adapter %d does not target slot %d", a, slots[k]);
            entry[(size_t)a * n_slots + k] = &ad->rec.targets[at];
        }
    }
    // segments: in range, disjoint
    std::vector<std::pair<int32_t, int32_t>> spans;
    for (int32_t i = 0; i < n_segs; ++i) {
        const tidal_lora_segment& g = segs[i];
        if (g.token_begin < 0 || g.token_end < g.token_begin || g.token_end > n_tokens)
            return fail(TIDAL_E_INVAL, "segment %d: tokens [%d, %d) outside 0..%d", i, g.token_begin, g.token_end,
                        n_tokens);
        if (g.adapter >= n_adapters) return fail(TIDAL_E_INVAL, "segment %d: adapter %d out of range", i, g.adapter);
        if (g.token_end > g.token_begin) spans.push_back({g.token_begin, g.token_end});
    }
    std::sort(spans.begin(), spans.end());
    for (size_t i = 1; i < spans.size(); ++i)
        if (spans[i].first < spans[i - 1].second)
            return fail(TIDAL_E_INVAL, "segments overlap at token %d", spans[i].first);

    // what there is to do: segments with an adapter, on slots that exist
    struct HostSeg { int32_t t0, t1, adapter; };
    std::vector<HostSeg> longs, shorts;
    for (int32_t i = 0; i < n_segs; ++i) {
        const tidal_lora_segment& g = segs[i];
        if (g.adapter < 0 || g.token_end == g.token_begin) continue;
        (g.token_end - g.token_begin <= kApplyShortRows ? shorts : longs).push_back(HostSeg{g.token_begin, g.token_end, g.adapter});
    }
    if (n_slots > kMaxApplySlots) return fail(TIDAL_E_INVAL, "at most %d slots per call", kMaxApplySlots);
    ApplySlot slot_tab[kMaxApplySlots];
    memset(slot_tab, 0, sizeof slot_tab);
    int max_out = 0;
    bool any = false;
    for (int32_t k = 0; k < n_slots; ++k) {
        const SlotState& st = t->slots[slots[k]];
        slot_tab[k].out = st.elems > 0 ? (int32_t)st.rows : 0;
        slot_tab[k].u_tok = (uint32_t)((int64_t)k * n_tokens);
        max_out = std::max(max_out, slot_tab[k].out);
    }
    // factors of an (adapter, slot) pair, as offsets from the lowest adapter address
    const char* lowest = nullptr;
    for (int32_t a = 0; a < n_adapters; ++a)
        if (!lowest || adapters[a]->rec.dev < lowest) lowest = adapters[a]->rec.dev;
    std::vector<char> used((size_t)std::max(n_adapters, 1), 0);
    for (const HostSeg& g : longs) used[g.adapter] = 1;
    for (const HostSeg& g : shorts) used[g.adapter] = 1;
    std::vector<ApplyFactor> facs((size_t)n_adapters * (size_t)std::max(n_slots, 1));
    for (int32_t a = 0; a < n_adapters; ++a) {
        for (int32_t k = 0; k < n_slots; ++k) {
            ApplyFactor& f = facs[(size_t)a * n_slots + k];
            memset(&f, 0, sizeof f);
            const PackedTarget* p = entry[(size_t)a * n_slots + k];
            if (!used[a] || slot_tab[k].out == 0 || !p->active()) continue;     // r stays 0: nothing to do
            if (p->ar_off == kNoOffset)
                return fail(TIDAL_E_STATE, "adapter %d holds no row-major A for slot %d", a, slots[k]);
            const uint64_t ar = (uint64_t)(adapters[a]->rec.dev - lowest) + p->ar_off;
            const uint64_t bp = (uint64_t)(adapters[a]->rec.dev - lowest) + p->bp_off;
            if (ar % kLoraUnit || bp % kLoraUnit || ar / kLoraUnit > 0xFFFFFFFFull || bp / kLoraUnit > 0xFFFFFFFFull)
                return fail(TIDAL_E_INVAL, "adapter %d lies too far from the others (more than 1 TB of address space)", a);
            f.ar = (uint32_t)(ar / kLoraUnit);
            f.bp = (uint32_t)(bp / kLoraUnit);
            f.s = p->alpha / (float)p->r;
            f.r = (uint16_t)p->r;
            f.rp = (uint16_t)p->rp;
            if (!ys || !ys[k]) return fail(TIDAL_E_INVAL, "y of slot %d is NULL", slots[k]);
            if ((uintptr_t)ys[k] % 16) return fail(TIDAL_E_INVAL, "y of slot %d is not 16-byte aligned", slots[k]);
            any = true;
        }
    }
    if (!any) return TIDAL_OK;
    for (int32_t k = 0; k < n_slots; ++k) slot_tab[k].y = (uint16_t*)(ys ? ys[k] : nullptr);
    if (!x) return fail(TIDAL_E_INVAL, "x is NULL");
    if ((uintptr_t)x % 16) return fail(TIDAL_E_INVAL, "x must be 16-byte aligned");
    if (!workspace || (uintptr_t)workspace % kSlotAlign) return fail(TIDAL_E_INVAL, "workspace is NULL or not 256-byte aligned");
    const int64_t ws_tokens = (int64_t)n_tokens * n_slots;
    if (ws_tokens > 0x7FFFFFFF) return fail(TIDAL_E_INVAL, "n_tokens x n_slots is too large");
    if (workspace_bytes < tidal_lora_apply_workspace_bytes((int32_t)ws_tokens))
        return fail(TIDAL_E_NOMEM, "workspace needs %zu bytes, got %zu", tidal_lora_apply_workspace_bytes((int32_t)ws_tokens),
                    workspace_bytes);
    // resident adapters exist, so their upload has set the template's device side up already; the
    // allocation-free entry point relies on that and creates nothing
    if (no_alloc && !t->dev_ready) return fail(TIDAL_E_STATE, "the template has not been used on a device yet");
    int rc = no_alloc ? TIDAL_OK : ensure_device(t);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_;
    for (int32_t a = 0; a < n_adapters; ++a) {                                       // the uploads of the adapters in use
        if (!used[a] || !adapters[a]->rec.ready || adapters[a]->upload_seen_done) continue;
        if (hipEventQuery(adapters[a]->rec.ready) == hipSuccess) {
            adapters[a]->upload_seen_done = true;                                    // finished uploads need no wait, now or later
            continue;
        }
        (void)hipGetLastError();                                                     // hipErrorNotReady is no error here
        HIP_TRY(hipStreamWaitEvent(stream, adapters[a]->rec.ready, 0));
    }

    // with ordered accumulation every segment takes the (slow, bit-reproducible) ordered kernels
    const bool ordered = (t->cfg.flags & TIDAL_FLAG_ORDERED_ACCUM) != 0;
    if (ordered) {
        longs.insert(longs.end(), shorts.begin(), shorts.end());
        shorts.clear();
    }
    // ---- prompts: one self-contained entry per (segment, active slot), kMaxApplyLong per launch
    std::vector<ApplyLongEntry> long_entries;
    for (const HostSeg& g : longs) {
        for (int32_t k = 0; k < n_slots; ++k) {
            const ApplyFactor& f = facs[(size_t)g.adapter * n_slots + k];
            if (f.r == 0) continue;
            ApplyLongEntry e;
            memset(&e, 0, sizeof e);
            e.Ar = (const uint16_t*)(lowest + (size_t)f.ar * kLoraUnit);
            e.Bp = (const uint16_t*)(lowest + (size_t)f.bp * kLoraUnit);
            e.y = slot_tab[k].y;
            e.t0 = g.t0;
            e.t1 = g.t1;
            e.s = f.s;
            e.r = f.r;
            e.rp = f.rp;
            e.out = slot_tab[k].out;
            e.u_tok = slot_tab[k].u_tok;
            long_entries.push_back(e);
        }
    }
    // shrink = true: u = bf16(A x) for all entries; else the expand of the entries with padded
    // rank rp (the specialised kernels run at twice the occupancy of the one that takes any rank)
    auto run_long = [&](bool shrink, int rp) -> int {
        std::vector<const ApplyLongEntry*> list;
        for (const ApplyLongEntry& e : long_entries)
            if (shrink || e.rp == rp) list.push_back(&e);
        for (size_t at = 0; at < list.size(); at += kMaxApplyLong) {
            const int n = (int)std::min(list.size() - at, (size_t)kMaxApplyLong);
            ApplyLongBatch b;
            memset(&b, 0, sizeof b);
            b.x = (const uint16_t*)x;
            b.u = (uint16_t*)workspace;
            b.n = n;
            int64_t tiles = 0;
            int launch_out = 0;
            for (int k = 0; k < n; ++k) {
                tiles += ((int64_t)list[at + k]->t1 - list[at + k]->t0 + 31) / 32;
                launch_out = std::max(launch_out, list[at + k]->out);
            }
            // tiles a wave walks per strip of B: long walks amortise the strip, short ones keep
            // small batches spread over the chip (aim: >= 1024 waves; measured best of 1, 2, 4)
            const int64_t strips = (launch_out + 255) / 256;
            int ct = (int)std::max<int64_t>(1, std::min<int64_t>(kApplyChunkTiles, tiles * strips / 1024));
            if (tuning_knobs().apply_ct >= 1) ct = tuning_knobs().apply_ct;      // tuning builds only
            int64_t units = 0;
            for (int k = 0; k < kMaxApplyLong; ++k) b.first[k] = 0x7FFFFFFF;
            for (int k = 0; k < n; ++k) {
                b.e[k] = *list[at + k];
                const int64_t len = (int64_t)b.e[k].t1 - b.e[k].t0;
                b.first[k] = (int32_t)units;
                units += shrink ? (len + 31) / 32 : (len + 32 * ct - 1) / (32 * ct);
            }
            if (units > 0x7FFFFFF0) return fail(TIDAL_E_INVAL, "batch too large");
            if (ordered) HIP_TRY(launch_apply_ordered(b, (int)in, shrink, stream));
            else if (shrink) HIP_TRY(launch_apply_shrink(b, (int)units, (int)in, stream));
            else HIP_TRY(launch_apply_expand(b, (int)units, ct, launch_out, rp, stream));
        }
        return TIDAL_OK;
    };
    // Default for prompts: both steps of a token tile in one workgroup, one launch per kMaxApplyLong
    // entries.  Batches too small to give every compute unit a 32-token tile take 16-token tiles.
    auto run_fused = [&]() -> int {
        int64_t tiles32 = 0;
        for (const ApplyLongEntry& e : long_entries) tiles32 += ((int64_t)e.t1 - e.t0 + 31) / 32;
        int tr = tiles32 < 256 ? 16 : 32;
        if (tuning_knobs().apply_tile_rows > 0) tr = tuning_knobs().apply_tile_rows;      // tuning builds only
        for (size_t at = 0; at < long_entries.size(); at += kMaxApplyLong) {
            const int n = (int)std::min(long_entries.size() - at, (size_t)kMaxApplyLong);
            ApplyLongBatch b;
            memset(&b, 0, sizeof b);
            b.x = (const uint16_t*)x;
            b.u = nullptr;                               // u never leaves the workgroup
            b.n = n;
            int64_t units = 0;
            for (int k = 0; k < kMaxApplyLong; ++k) b.first[k] = 0x7FFFFFFF;
            for (int k = 0; k < n; ++k) {
                b.e[k] = long_entries[at + k];
                b.first[k] = (int32_t)units;
                units += ((int64_t)b.e[k].t1 - b.e[k].t0 + tr - 1) / tr;
            }
            if (units > 0x7FFFFFF0) return fail(TIDAL_E_INVAL, "batch too large");
            HIP_TRY(launch_apply_fused(b, (int)units, tr, (int)in, stream));
        }
        return TIDAL_OK;
    };
    // ---- decode steps: compact tables, up to kMaxApplyShort segments whose adapters' factor
    // entries (n_slots each) fit the factor table
    auto run_short = [&](bool shrink) -> int {
        size_t at = 0;
        while (at < shorts.size()) {
            ApplyShortBatch b;
            memset(&b, 0, sizeof b);
            b.x = (const uint16_t*)x;
            b.u = (uint16_t*)workspace;
            b.adapter_base = lowest;
            b.n_slots = n_slots;
            memcpy(b.slot, slot_tab, sizeof slot_tab);
            std::vector<int> fac_of((size_t)std::max(n_adapters, 1), -1);      // adapter -> its first factor entry of this launch
            int n = 0, nfac = 0;
            while (at + n < shorts.size() && n < kMaxApplyShort) {
                const HostSeg& g = shorts[at + n];
                if (fac_of[g.adapter] < 0) {
                    if (nfac + n_slots > kMaxApplyFactors) break;
                    fac_of[g.adapter] = nfac;
                    for (int32_t k = 0; k < n_slots; ++k) b.fac[nfac + k] = facs[(size_t)g.adapter * n_slots + k];
                    nfac += n_slots;
                }
                b.seg[n].t0 = g.t0;
                b.seg[n].rows = (uint16_t)(g.t1 - g.t0);
                b.seg[n].fac = (uint16_t)fac_of[g.adapter];
                ++n;
            }
            b.n_segs = n;
            if (shrink) HIP_TRY(launch_apply_shrink_short(b, (int)in, stream));
            else HIP_TRY(launch_apply_expand_short(b, max_out, stream));
            at += n;
        }
        return TIDAL_OK;
    };
    const bool two_step = ordered || tuning_knobs().apply_two_step == 1;      // the knob: tuning builds only
    // Decode segments stay two launches: one workgroup per (request, target) that computes all of u
    // itself was tried and lost (35 instead of 20 us for 64 requests: a single compute unit cannot
    // pull a 64-rank A through fast enough), and the shrink of a request must be spread over many
    // compute units, which puts a grid-wide dependency in front of the expand.  The prompts' launch
    // goes in between and covers the hand-over.
    rc = run_short(true);
    if (rc) return rc;
    rc = two_step ? run_long(true, 0) : run_fused();
    if (rc) return rc;
    if (two_step)
        for (int rp = 16; rp <= 64; rp *= 2) {
            rc = run_long(false, rp);
            if (rc) return rc;
        }
    rc = run_short(false);
    host_call_report(64);
    return rc;
}

extern "C" int tidal_lora_apply(tidal_template* t, int32_t slot, const tidal_adapter* const* adapters,
                                int32_t n_adapters, const tidal_lora_segment* segs, int32_t n_segs, const void* x,
                                void* y, int32_t n_tokens, void* workspace, size_t workspace_bytes, void* stream) {
    void* ys[1] = {y};
    return lora_apply_impl(t, &slot, 1, adapters, n_adapters, segs, n_segs, x, ys, n_tokens, workspace, workspace_bytes,
                           stream);
}

extern "C" int32_t tidal_lora_apply_static_max_tokens(void) { return kStaticApplyTokens; }

extern "C" int tidal_lora_apply_static(tidal_template* t, int32_t slot, const tidal_adapter* const* adapters,
                                       int32_t n_adapters, const tidal_lora_segment* segs, int32_t n_segs,
                                       const void* x, void* y, int32_t n_tokens, void* stream) {
    if (n_tokens > kStaticApplyTokens)
        return fail(TIDAL_E_INVAL, "n_tokens = %d exceeds the %d token rows the library's scratch memory holds; "
                    "use tidal_lora_apply with a workspace", n_tokens, kStaticApplyTokens);
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    void* ws = nullptr;
    if (dev >= 0 && dev < kMaxDevices) {
        std::lock_guard<std::mutex> lock(g_scratch_mu);
        ws = g_scratch_ptr[dev];
    }
    if (!ws) return fail(TIDAL_E_STATE, "no template has been set up on device %d yet (adapters are uploaded first)", dev);
    void* ys[1] = {y};
    return lora_apply_impl(t, &slot, 1, adapters, n_adapters, segs, n_segs, x, ys, n_tokens, ws, kStaticScratchBytes,
                           stream, true);
}

extern "C" int tidal_lora_apply_multi(tidal_template* t, const int32_t* slots, int32_t n_slots,
                                      const tidal_adapter* const* adapters, int32_t n_adapters,
                                      const tidal_lora_segment* segs, int32_t n_segs, const void* x, void* const* ys,
                                      int32_t n_tokens, void* workspace, size_t workspace_bytes, void* stream) {
    return lora_apply_impl(t, slots, n_slots, adapters, n_adapters, segs, n_segs, x, ys, n_tokens, workspace,
                           workspace_bytes, stream);
}

extern "C" int tidal_lora_detach(tidal_template* t, void* stream) {
    if (!t) return fail(TIDAL_E_INVAL, "template is NULL");
    if (!t->attached) return fail(TIDAL_E_STATE, "no adapter is attached");
    int rc = ensure_device(t);
    if (rc) return rc;
    AdapterRec old = t->cur;
    rc = launch_rmw(t, &old, nullptr, (hipStream_t)stream);
    if (rc) return rc;
    if (t->cur_resident) t->cur_resident->attached = false;
    t->attached = false;
    t->cur_resident = nullptr;
    // cur_region keeps its value: the next host-pointer attach then uses the other region,
    // so a still-running detach kernel never has its factors overwritten
    t->cur.targets.clear();
    return TIDAL_OK;
}

// ---------------------------------------------------------------------------------------
// copy-on-write forks
// ---------------------------------------------------------------------------------------
struct tidal_fork {
    tidal_template* t;
    std::vector<int32_t> slots;      // sorted
    std::vector<size_t> offset;      // byte offset of each slot's private copy in dev
    char* dev;
    size_t bytes;
};

static int fork_layout(const tidal_template* t, const int32_t* slots, int32_t n, std::vector<int32_t>* sl,
                       std::vector<size_t>* off, size_t* total) {
    if (!t) return fail(TIDAL_E_INVAL, "template is NULL");
    if (n < 0 || (!slots && n > 0)) return fail(TIDAL_E_INVAL, "bad slot list (n=%d)", n);
    sl->assign(slots, slots + n);
    std::sort(sl->begin(), sl->end());
    size_t o = 0;
    off->clear();
    for (int32_t i = 0; i < n; ++i) {
        const int32_t s = (*sl)[i];
        if (s < 0 || s >= (int32_t)t->slots.size()) return fail(TIDAL_E_INVAL, "slot %d out of range", s);
        if (i > 0 && s == (*sl)[i - 1]) return fail(TIDAL_E_INVAL, "slot %d given twice", s);
        off->push_back(o);
        o = align_up(o + 2 * (size_t)t->slots[s].elems, kSlotAlign);
    }
    *total = o ? o : kSlotAlign;
    return TIDAL_OK;
}

extern "C" size_t tidal_fork_required_bytes(const tidal_template* t, const int32_t* slots, int32_t n) {
    std::vector<int32_t> sl;
    std::vector<size_t> off;
    size_t total = 0;
    if (fork_layout(t, slots, n, &sl, &off, &total)) return 0;
    return total;
}

extern "C" int tidal_fork_create(tidal_template* t, const int32_t* slots, int32_t n, void* dev_mem, size_t dev_bytes,
                                 tidal_fork** out) {
    if (!out) return fail(TIDAL_E_INVAL, "out is NULL");
    *out = nullptr;
    std::vector<int32_t> sl;
    std::vector<size_t> off;
    size_t total = 0;
    int rc = fork_layout(t, slots, n, &sl, &off, &total);
    if (rc) return rc;
    if (!dev_mem) return fail(TIDAL_E_INVAL, "dev_mem is NULL");
    if ((uintptr_t)dev_mem % kSlotAlign) return fail(TIDAL_E_INVAL, "dev_mem is not 256-byte aligned");
    if (total > dev_bytes) return fail(TIDAL_E_NOMEM, "fork needs %zu bytes, got %zu", total, dev_bytes);
    if (total / kLoraUnit > 0xFFFFFFFFull) return fail(TIDAL_E_INVAL, "fork too large");
    tidal_fork* f = new (std::nothrow) tidal_fork();
    if (!f) return fail(TIDAL_E_NOMEM, "out of host memory");
    f->t = t;
    f->slots = sl;
    f->offset = off;
    f->dev = (char*)dev_mem;
    f->bytes = total;
    *out = f;
    return TIDAL_OK;
}

extern "C" int tidal_fork_destroy(tidal_fork* f) {
    delete f;
    return TIDAL_OK;
}

extern "C" int tidal_fork_slot_ptr(const tidal_fork* f, int32_t slot, void** dev_ptr, size_t* bytes) {
    if (!f || !dev_ptr) return fail(TIDAL_E_INVAL, "NULL argument");
    auto it = std::lower_bound(f->slots.begin(), f->slots.end(), slot);
    if (it == f->slots.end() || *it != slot) return fail(TIDAL_E_INVAL, "slot %d is not part of this fork", slot);
    *dev_ptr = f->dev + f->offset[(size_t)(it - f->slots.begin())];
    if (bytes) *bytes = 2 * (size_t)f->t->slots[slot].elems;
    return TIDAL_OK;
}

extern "C" int tidal_fork_apply(tidal_fork* f, const tidal_adapter* a, void* stream_) {
    if (!f) return fail(TIDAL_E_INVAL, "fork is NULL");
    tidal_template* t = f->t;
    hipStream_t stream = (hipStream_t)stream_;
    if (a && a->owner != t) return fail(TIDAL_E_INVAL, "adapter belongs to another template");
    if (t->attached) return fail(TIDAL_E_STATE, "an adapter is merged into the template in place; detach it first");
    for (int32_t s : f->slots)
        if (!t->slots[s].materialised && t->slots[s].elems > 0)
            return fail(TIDAL_E_STATE, "fork slot %d was never materialised", s);
    std::map<int32_t, const PackedTarget*> active;
    if (a)
        for (const PackedTarget& p : a->rec.targets) {
            if (!std::binary_search(f->slots.begin(), f->slots.end(), p.slot))
                return fail(TIDAL_E_INVAL, "adapter targets slot %d, which is not part of the fork", p.slot);
            if (p.active() && t->slots[p.slot].elems > 0) active[p.slot] = &p;
        }
    int rc = ensure_device(t);
    if (rc) return rc;
    rc = wait_marks(t, kMarkLoad, stream);
    if (rc) return rc;
    rc = wait_marks(t, kMarkLora, stream);       // a detach that restored the template on another stream
    if (rc) return rc;
    if (a && a->rec.ready) HIP_TRY(hipStreamWaitEvent(stream, a->rec.ready, 0));
    std::map<LoraKey, std::vector<LoraTargetDev>> groups;
    for (size_t i = 0; i < f->slots.size(); ++i) {
        const int32_t slot = f->slots[i];
        const SlotState& s = t->slots[slot];
        if (s.elems == 0) continue;
        auto it = active.find(slot);
        if (it == active.end()) {
            // not written by this adapter: the private copy is the template's value again
            HIP_TRY(hipMemcpyAsync(f->dev + f->offset[i], slot_ptr(t, slot), 2 * (size_t)s.elems, hipMemcpyDeviceToDevice, stream));
            continue;
        }
        const PackedTarget* p = it->second;
        LoraTargetDev d;
        memset(&d, 0, sizeof d);
        if (t->lay.slot_offset[slot] / kLoraUnit > 0xFFFFFFFFull)
            return fail(TIDAL_E_INVAL, "slot %d lies beyond 1 TB from the start of the arena", slot);
        d.w = (uint32_t)(t->lay.slot_offset[slot] / kLoraUnit);
        d.at_old = (uint32_t)(f->offset[i] / kLoraUnit);               // destination, relative to the fork's memory
        d.at_new = (uint32_t)(p->at_off / kLoraUnit);
        d.bp_new = (uint32_t)(p->bp_off / kLoraUnit);
        d.s_new = p->alpha / (float)p->r;
        groups[LoraKey(s.rows, s.cols, 0, p->rp, 0, p->r)].push_back(d);
        t->stats.rmw_elems += (uint64_t)s.elems;
    }
    rc = launch_groups(t, groups, f->dev, a ? a->rec.dev : nullptr, true, stream);
    if (rc) return rc;
    return mark_done(t, kMarkLora, stream);
}

// ---------------------------------------------------------------------------------------
// partial residency (Sec. 5.2, Eq. 1) and the stand-in consumer
// ---------------------------------------------------------------------------------------
extern "C" size_t tidal_prefetch_bytes(size_t model_bytes, double ttft_seconds, double link_bytes_per_second) {
    if (!(ttft_seconds >= 0.0) || !(link_bytes_per_second >= 0.0)) return 0;
    const double hidden = ttft_seconds * link_bytes_per_second;      // bytes that stream in under the inference
    if (!(hidden < (double)model_bytes)) return 0;
    const double need = (double)model_bytes - hidden;
    size_t r = (size_t)need;
    if ((double)r < need) ++r;                                       // round up: never prefetch too little
    return r > model_bytes ? model_bytes : r;
}

extern "C" int tidal_template_resident_prefix(const tidal_template* t, size_t prefetch_bytes, int32_t* n_slots,
                                              size_t* bytes) {
    if (!t || !n_slots) return fail(TIDAL_E_INVAL, "NULL argument");
    size_t sum = 0;
    int32_t n = 0;
    // smallest prefix that covers prefetch_bytes (residency is slot-granular, so round up)
    while (n < (int32_t)t->slots.size() && sum < prefetch_bytes) {
        sum += 2 * (size_t)t->slots[n].elems;
        ++n;
    }
    *n_slots = n;
    if (bytes) *bytes = sum;
    return TIDAL_OK;
}

extern "C" int tidal_slot_checksum(tidal_template* t, int32_t slot, int32_t passes, void* stream, uint64_t* dev_sum) {
    if (!t || !dev_sum) return fail(TIDAL_E_INVAL, "NULL argument");
    if (slot < 0 || slot >= (int32_t)t->slots.size()) return fail(TIDAL_E_INVAL, "slot %d out of range", slot);
    if (passes < 1 || passes > (1 << 20)) return fail(TIDAL_E_INVAL, "passes outside 1..2^20");
    if ((uintptr_t)dev_sum % 8) return fail(TIDAL_E_INVAL, "dev_sum is not 8-byte aligned");
    SlotState& s = t->slots[slot];
    if (s.elems == 0) return TIDAL_OK;
    if (!s.materialised) return fail(TIDAL_E_STATE, "slot %d was never materialised", slot);
    if ((t->cfg.flags & TIDAL_FLAG_SLOT_EVENTS) && s.ready_recorded)
        HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, s.ready, 0));
    HIP_TRY(launch_slot_checksum(slot_ptr(t, slot), s.elems, passes, dev_sum, (hipStream_t)stream));
    return TIDAL_OK;
}

// ---------------------------------------------------------------------------------------
// utilities
// ---------------------------------------------------------------------------------------
extern "C" int tidal_convert_device(void* dst_bf16, const void* src, int32_t dtype, int64_t n, void* stream) {
    if (n < 0) return fail(TIDAL_E_INVAL, "n is negative");
    if (n == 0) return TIDAL_OK;
    if (!dst_bf16 || !src) return fail(TIDAL_E_INVAL, "NULL argument");
    if (!dtype_ok(dtype)) return fail(TIDAL_E_INVAL, "unknown dtype %d", dtype);
    if ((uintptr_t)dst_bf16 % 16 || (uintptr_t)src % 16) return fail(TIDAL_E_INVAL, "pointers must be 16-byte aligned");
    ConvertBatch batch;
    batch.seg[0] = ConvertSegment{src, dst_bf16, n, dtype, 0};
    HIP_TRY(launch_convert(batch, 1, (hipStream_t)stream));
    return TIDAL_OK;
}

extern "C" int tidal_h2d_peak(void* dev, size_t bytes, int32_t reps, void* stream, double* gbytes_per_s) {
    if (!dev || !gbytes_per_s || bytes == 0 || reps <= 0) return fail(TIDAL_E_INVAL, "bad argument");
    char* host = nullptr;
    HIP_TRY(hipHostMalloc((void**)&host, bytes, hipHostMallocDefault));
    memset(host, 1, bytes);
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t e = hipEventCreate(&a);
    if (e == hipSuccess) e = hipEventCreate(&b);
    double best = 0.0;
    hipStream_t s = (hipStream_t)stream;
    for (int i = 0; i < reps + 1 && e == hipSuccess; ++i) {     // first pass is a warm-up
        e = hipEventRecord(a, s);
        if (e == hipSuccess) e = hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipEventRecord(b, s);
        if (e == hipSuccess) e = hipEventSynchronize(b);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
        if (e == hipSuccess && i > 0 && ms > 0.f) best = std::max(best, (double)bytes / (ms * 1e-3) / 1e9);
    }
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    (void)hipHostFree(host);
    if (e != hipSuccess) return fail(TIDAL_E_HIP, "h2d probe failed: %s", hipGetErrorString(e));
    *gbytes_per_s = best;
    return TIDAL_OK;
}

extern "C" int tidal_hbm_probe(void* dev, int64_t rows, int64_t cols, int64_t n, int32_t blocks_per_walk, int32_t mode,
                               int32_t reps, void* stream, double* gbytes_per_s) {
    if (!dev || !gbytes_per_s || reps <= 0) return fail(TIDAL_E_INVAL, "bad argument");
    if (rows <= 0 || cols <= 0 || n <= 0 || rows % 32 || cols % 256 || rows > 0x7FFFFFFF || cols > 0x7FFFFFFF)
        return fail(TIDAL_E_INVAL, "rows must be a positive multiple of 32 and cols of 256");
    if (blocks_per_walk < 1 || blocks_per_walk > 1024) return fail(TIDAL_E_INVAL, "blocks_per_walk outside 1..1024");
    if (mode < TIDAL_PROBE_RMW || mode > TIDAL_PROBE_WRITE) return fail(TIDAL_E_INVAL, "unknown probe mode %d", mode);
    if ((uintptr_t)dev % 16) return fail(TIDAL_E_INVAL, "dev is not 16-byte aligned");
    const double bytes_per_elem = mode == TIDAL_PROBE_RMW ? 4.0 : 2.0;
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t e = hipEventCreate(&a);
    if (e == hipSuccess) e = hipEventCreate(&b);
    hipStream_t s = (hipStream_t)stream;
    double best = 0.0;
    for (int i = 0; i < reps + 1 && e == hipSuccess; ++i) {     // first pass is a warm-up
        e = hipEventRecord(a, s);
        if (e == hipSuccess) e = launch_rmw_probe(dev, rows, cols, n, blocks_per_walk, mode, s);
        if (e == hipSuccess) e = hipEventRecord(b, s);
        if (e == hipSuccess) e = hipEventSynchronize(b);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
        if (e == hipSuccess && i > 0 && ms > 0.f)
            best = std::max(best, bytes_per_elem * (double)rows * (double)cols * (double)n / (ms * 1e-3) / 1e9);
    }
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    if (e != hipSuccess) return fail(TIDAL_E_HIP, "memory probe failed: %s", hipGetErrorString(e));
    *gbytes_per_s = best;
    return TIDAL_OK;
}

extern "C" int tidal_hbm_rmw_peak(void* dev, int64_t rows, int64_t cols, int64_t n, int32_t blocks_per_walk, int32_t reps,
                                  void* stream, double* gbytes_per_s) {
    return tidal_hbm_probe(dev, rows, cols, n, blocks_per_walk, TIDAL_PROBE_RMW, reps, stream, gbytes_per_s);
}

extern "C" int tidal_get_stats(tidal_template* t, tidal_stats* out) {
    if (!t || !out) return fail(TIDAL_E_INVAL, "NULL argument");
    int rc = timing_drain(t);
    if (rc) return rc;
    *out = t->stats;
    return TIDAL_OK;
}

extern "C" int tidal_reset_stats(tidal_template* t) {
    if (!t) return fail(TIDAL_E_INVAL, "template is NULL");
    int rc = timing_drain(t);
    if (rc) return rc;
    memset(&t->stats, 0, sizeof t->stats);
    return TIDAL_OK;
}

extern "C" int tidal_template_sync(tidal_template* t) {
    if (!t) return fail(TIDAL_E_INVAL, "template is NULL");
    if (!t->dev_ready) return TIDAL_OK;
    for (StreamMark& m : t->marks)
        if (m.active) {
            HIP_TRY(hipEventSynchronize(m.ev));
            m.active = false;
        }
    return TIDAL_OK;
}

extern "C" int tidal_template_destroy(tidal_template* t) {
    if (!t) return TIDAL_OK;
    int rc = tidal_template_sync(t);
    if (t->dev_ready) {
        for (const auto& m : t->load_marks) (void)hipEventDestroy(m.done);
        for (hipEvent_t e : t->load_mark_pool) (void)hipEventDestroy(e);
        for (int b = 0; b < 2; ++b) {
            if (t->bounce_used[b]) (void)hipEventSynchronize(t->bounce_free[b]);
            (void)hipEventDestroy(t->staged_ready[b]);
            (void)hipEventDestroy(t->staging_free[b]);
            (void)hipEventDestroy(t->bounce_free[b]);
            if (t->bounce[b]) (void)hipHostFree(t->bounce[b]);
        }
        if (t->up_stream) {
            (void)hipStreamSynchronize(t->up_stream);
            for (int g = 0; g < kMaxUploadGroups; ++g) {
                (void)hipEventDestroy(t->ev_group_copied[g]);
                (void)hipEventDestroy(t->ev_group_packed[g]);
            }
            (void)hipEventDestroy(t->ev_up_begin);
            for (int k = 0; k < 4; ++k) (void)hipEventDestroy(t->rates.ev[k]);
            (void)hipStreamDestroy(t->up_stream);
        }
        (void)hipEventDestroy(t->ev_start);
        (void)hipEventDestroy(t->ev_copy_done);
        for (StreamMark& m : t->marks) (void)hipEventDestroy(m.ev);
        for (SlotState& s : t->slots)
            if (s.ready) (void)hipEventDestroy(s.ready);
        (void)timing_drain(t);
        for (hipEvent_t e : t->timing_pool) (void)hipEventDestroy(e);
    }
    if (t->cur_resident) t->cur_resident->attached = false;
    delete t;
    return rc;
}

extern "C" const char* tidal_last_error(void) { return g_err; }
