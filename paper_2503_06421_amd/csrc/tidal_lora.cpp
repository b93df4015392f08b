// libtidal host side, part two: adapters (validation, packed layout, upload), the attach / swap /
// detach state machine with its grouped upload, and copy-on-write forks.
#include <map>
#include <new>
#include <tuple>

#include "tidal_host.h"

using namespace tidal;

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

    // A small adapter whose factors lie in pinned memory is not staged at all: pinned host memory is mapped
    // into the GPU's address space, so the pack kernel reads the factors over the link itself, every element
    // once, in 16-byte pieces -- one launch less than copy + pack (single 4096 x 4096 layer, r = 8: attach
    // from host pointers 45 -> 37 us).  Factors the pack kernel would take element by element (odd ranks or
    // widths, unaligned) are staged as before: single elements are no way to cross the link.
    {
        size_t total = 0;
        bool direct = true;
        for (const Job& j : jobs) {
            total += j.bytes;
            const bool vec = j.seg.layout == kPackAt ? j.seg.lines % 8 == 0 : j.seg.r % 8 == 0;
            direct = direct && j.pinned && vec && (uintptr_t)j.host % 16 == 0;
        }
        std::vector<PackSegment> segs;
        for (size_t k = 0; direct && total <= kKernelCopyMax && k < jobs.size(); ++k) {
            void* view = nullptr;
            if (HIP_TIMED(hipHostGetDevicePointer(&view, const_cast<char*>(jobs[k].host), 0)) != hipSuccess || !view ||
                (uintptr_t)view % 16 != 0) {
                (void)hipGetLastError();
                direct = false;
                break;
            }
            PackSegment sg = jobs[k].seg;
            sg.src = view;
            segs.push_back(sg);
            if (jobs[k].has2) {
                sg = jobs[k].seg2;
                sg.src = view;
                segs.push_back(sg);
            }
        }
        if (direct && total <= kKernelCopyMax) {
            t->stats.h2d_bytes += total;
            return launch_packs(segs, pack);
        }
    }

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
int tidal::launch_rmw(tidal_template* t, const AdapterRec* older, const AdapterRec* newer, hipStream_t stream) {
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
    constexpr double kLaunchMs = 0.045;            // what one more launch costs: its bubble, its ramp and tail (70B-shaped adapter, 16 to 28 launches)
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
    const double pack_rate = 2.0e9;                                      // bytes per ms through the pack kernel
    const double group_cap = 0.5 * (double)staging_span(t);              // a group's factors: half the staging memory, so that
                                                                         // the next group's copies need not wait for its packs
    static const double kGrowth[] = {1.0, 1.5, 2.0, 3.0};
    static const double kFirst[] = {1.0, 0.35};                           // the first group may be smaller still
    // Simulate a candidate on three resources -- the link, the packing stream, the caller's stream -- and keep
    // it if it ends first.  The link carries the groups back to back, as soon as the calling thread has got to
    // them; the caller's stream takes each group when its copies are in: pack, then merge (the first group's
    // copies run on the caller's stream and share the link with the second's).
    auto consider = [&](const std::vector<std::pair<size_t, size_t>>& cand) {
        if (cand.size() < 2 || cand.size() > (size_t)kMaxUploadGroups) return;
        double link_done = kWaitMs, merge_done = 0.0;
        bool fits = true, first_group = true;
        for (const auto& gr : cand) {
            double ug = 0.0, mg = 0.0, bytes = 0.0;
            for (size_t i = gr.first; i < gr.second; ++i) { ug += u[i]; mg += m[i]; bytes += raw[i]; }
            fits = fits && bytes <= group_cap;
            link_done += ug;                                 // the link's total does not depend on who shares it
            const double here = first_group ? 1.5 * ug : link_done + kHandoverMs;
            merge_done = std::max(merge_done, here) + 2.0 * bytes / pack_rate + mg + kGroupMs +
                         kLaunchMs * (launches(gr.first, gr.second) - 1);
            first_group = false;
        }
        if (fits && merge_done < best) {
            best = merge_done;
            best_groups = cand;
        }
    };
    // Family one: G groups whose shares of the upload grow by a factor q from one to the next (q = 1: equal
    // groups, what an upload-bound adapter wants; q > 1: a small first group, so that merging starts early,
    // and large later ones that hide under the merges before them).
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
            consider(cand);
        }
    }
    // Family two, for adapters of several times the staging memory whose merges outlast their upload: a small
    // first group, growth by q until a group reaches what the staging memory takes at a time, groups of that
    // size from there on (on the 70B-shaped adapter 8 / 40 / 160 / 176 / 176 targets measure 43.4 ms per
    // attach, seven near-equal groups 44.6).
    static const double kStart[] = {1.0 / 128, 1.0 / 64, 1.0 / 32, 1.0 / 16};
    static const double kSteep[] = {3.0, 4.0, 5.0};
    double raw_total = 0.0;
    for (size_t i = 0; i < n; ++i) raw_total += raw[i];
    for (double start : kStart)
        for (double q : kSteep) {
            std::vector<std::pair<size_t, size_t>> cand;
            size_t a0 = 0;
            double want = start * raw_total;
            while (a0 < n && cand.size() <= (size_t)kMaxUploadGroups) {
                const double lim = std::min(want, group_cap);
                size_t b0 = a0;
                double acc = 0.0;
                while (b0 < n && (acc + raw[b0] <= lim || b0 == a0)) acc += raw[b0++];
                cand.push_back({a0, b0});
                a0 = b0;
                want *= q;
            }
            if (a0 == n) consider(cand);
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

extern "C" int32_t tidal_lora_upload_plan(tidal_template* t, const tidal_lora_target* targets, int32_t n_targets,
                                          int32_t swap, int32_t* group_targets, int32_t cap) {
    AdapterRec rec;
    int rc = validate_targets(t, targets, n_targets, true, &rec);
    if (rc) return rc;
    if (cap < 0 || (!group_targets && cap > 0)) return fail(TIDAL_E_INVAL, "bad output buffer");
    std::vector<std::pair<size_t, size_t>> groups;
    const AdapterRec old = t->cur;
    plan_upload_groups(t, targets, rec, (swap && t->attached) ? &old : nullptr, &groups);
    for (size_t g = 0; g < groups.size() && (int32_t)g < cap; ++g)
        group_targets[g] = (int32_t)(groups[g].second - groups[g].first);
    return (int32_t)groups.size();
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

