// libtidal host side, part one: error reporting, templates (configuration, creation, slots), the
// two-stream staging pipeline of materialisation, partial residency and the measurement utilities.
// All arithmetic on tensor data happens in the kernels (convert_kernels.hip, lora_kernels.hip);
// this file only moves bytes and launches.
#include <new>
#include <thread>

#include "tidal_host.h"

using namespace tidal;

// ---------------------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------------------
static thread_local char g_err[512] = "";

int tidal::fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

// ---------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------
int tidal::ensure_device(tidal_template* t) {
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
int tidal::mark_done(tidal_template* t, int kind, hipStream_t stream) {
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
int tidal::wait_marks(tidal_template* t, int kind, hipStream_t stream) {
    for (const StreamMark& m : t->marks)
        if (m.active && m.kind == kind && m.stream != stream) HIP_TRY(hipStreamWaitEvent(stream, m.ev, 0));
    return TIDAL_OK;
}

int tidal::ensure_bounce(tidal_template* t, int b) {
    if (!t->bounce[b]) HIP_TRY(hipHostMalloc((void**)&t->bounce[b], t->cfg.chunk_bytes, hipHostMallocDefault));
    return TIDAL_OK;
}

int tidal::ensure_upload_stream(tidal_template* t) {
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
int tidal::timing_begin(tidal_template* t, hipStream_t s, hipEvent_t* start) {
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

int tidal::timing_end(tidal_template* t, hipStream_t s, hipEvent_t start, bool lora) {
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

bool tidal::host_is_pinned(const void* p) {
    hipPointerAttribute_t attr;
    hipError_t e = HIP_TIMED(hipPointerGetAttributes(&attr, p));
    if (e != hipSuccess) {
        (void)hipGetLastError();   // plain malloc'ed memory is reported as an error, not a type
        return false;
    }
    return attr.type == hipMemoryTypeHost;
}


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
void tidal::gather_copy(char* dst, const char* src, size_t bytes, int threads) {
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

int tidal::gather_sources(const tidal_template* t, const tidal_src* srcs, int32_t n_src, int32_t assume_pinned,
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
int tidal::check_rematerialise(const tidal_template* t, const std::vector<SourceInfo>& srcs, bool* clears) {
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

// The streaming loop.  `fuse` (optional): an adapter already packed on the device whose delta is
// added to its targets' slots while they are written (one rounding from the source).
int tidal::materialize_impl(tidal_template* t, std::vector<SourceInfo>& infos, bool clears, void* copy_stream,
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
