// libtidal host side, part three: adapters applied unmerged to a mixed batch, and the scratch memory
// of the entry point that allocates nothing.
#include <mutex>

#include "tidal_host.h"

using namespace tidal;

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
int tidal::resolve_scratch() {
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

