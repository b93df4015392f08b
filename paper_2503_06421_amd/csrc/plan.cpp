// Host-only planning for libtidal: configuration defaults, arena layout, copy plan.
#include "plan.h"

#include <stdlib.h>

#include <algorithm>

#include "tidal_internal.h"

namespace tidal {

bool normalise_config(const tidal_config* in, tidal_config* out, const char** msg) {
    tidal_config c;
    if (in) {
        c = *in;
    } else {
        c.chunk_bytes = 0;
        c.max_rank = 0;
        c.max_adapter_bytes = 0;
        c.flags = 0;
        c.coalesce_bytes = 0;
        c.gather_threads = 0;
        c.chunks_ahead = 0;
    }
    if (c.chunk_bytes == 0) c.chunk_bytes = (size_t)128 << 20;
    if (c.max_rank == 0) c.max_rank = 64;
    if (c.coalesce_bytes == 0) c.coalesce_bytes = (size_t)64 << 10;
    if (c.gather_threads == 0) c.gather_threads = 4;
    c.chunk_bytes = align_up(c.chunk_bytes, 4096);
    // the smaller the chunks, the fewer of them may queue up before the transfer rate suffers; and whatever
    // their size, from about 200 staged chunks in flight on every copy runs 6 % slower (two loads of 101
    // chunks of 128 MiB queued back to back: 254 ms each against 239)
    if (c.chunks_ahead == 0) c.chunks_ahead = (int32_t)std::min<size_t>(160, std::max<size_t>(16, c.chunk_bytes / ((size_t)800 << 10)));
    c.max_adapter_bytes = align_up(c.max_adapter_bytes, kSlotAlign);
    if (c.chunk_bytes < ((size_t)64 << 10)) { *msg = "chunk_bytes below 64 KiB"; return false; }
    if (c.chunk_bytes > ((size_t)1 << 32)) { *msg = "chunk_bytes above 4 GiB"; return false; }
    if (c.max_rank < 0 || c.max_rank > 64) { *msg = "max_rank outside 1..64"; return false; }
    if (c.coalesce_bytes > c.chunk_bytes) { *msg = "coalesce_bytes above chunk_bytes"; return false; }
    if (c.gather_threads < 1 || c.gather_threads > 16) { *msg = "gather_threads outside 1..16"; return false; }
    if (c.chunks_ahead < 1 || c.chunks_ahead > 4096) { *msg = "chunks_ahead outside 1..4096"; return false; }
    const int32_t known = TIDAL_FLAG_ORDERED_ACCUM | TIDAL_FLAG_TWO_PASS_SWAP | TIDAL_FLAG_SLOT_EVENTS |
                          TIDAL_FLAG_KERNEL_TIMING | TIDAL_FLAG_ASYNC_ENQUEUE | TIDAL_FLAG_NO_COPY_MERGE |
                          TIDAL_FLAG_PIPELINED_UPLOAD | TIDAL_FLAG_SERIAL_UPLOAD;
    if (c.flags & ~known) { *msg = "unknown flag bits"; return false; }
    *out = c;
    return true;
}

bool layout_arena(const tidal_slot_desc* slots, int32_t n, const tidal_config& cfg, ArenaLayout* out) {
    out->slot_offset.assign((size_t)n + 1, 0);
    size_t off = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (slots[i].rows < 0 || slots[i].cols < 0) return false;
        // guard the products against overflow: 2^46 elements per slot is far above any GPU
        if (slots[i].rows > ((int64_t)1 << 31) || slots[i].cols > ((int64_t)1 << 31)) return false;
        const uint64_t elems = (uint64_t)slots[i].rows * (uint64_t)slots[i].cols;
        if (elems > ((uint64_t)1 << 46)) return false;
        out->slot_offset[i] = off;
        off = align_up(off + 2 * (size_t)elems, kSlotAlign);
        if (off > ((size_t)1 << 50)) return false;
    }
    out->slot_offset[n] = off;
    out->staging[0] = off;
    out->staging[1] = off + cfg.chunk_bytes;
    off += 2 * cfg.chunk_bytes;
    out->adapter_region[0] = off;
    out->adapter_region[1] = off + cfg.max_adapter_bytes;
    off += 2 * cfg.max_adapter_bytes;
    out->total = off;
    return true;
}

void plan_copies(const std::vector<SourceInfo>& srcs, const tidal_config& cfg, int max_segments_per_chunk,
                 std::vector<Piece>* out) {
    out->clear();
    int32_t chunk = 0;
    size_t fill = 0;        // bytes of the current chunk's buffer in use
    int nseg = 0;           // staged (to be converted) pieces in the current chunk
    bool used = false;      // current chunk has at least one piece
    const size_t cap = cfg.chunk_bytes;

    for (const SourceInfo& s : srcs) {
        if (s.elems == 0) continue;
        const int64_t isz = (int64_t)dtype_size(s.dtype);
        const int64_t bytes = s.elems * isz;
        const bool gathered = !s.pinned || ((size_t)bytes < cfg.coalesce_bytes && !(cfg.flags & TIDAL_FLAG_NO_COPY_MERGE));
        const bool staged = s.dtype != TIDAL_BF16;
        int64_t remaining = s.elems, eoff = 0;

        if (!staged && !gathered) {
            // pinned bf16: DMA straight into the slot, no buffer; still cut at chunk size so a
            // single command never monopolises the copy queue for long
            const int64_t per = (int64_t)(cap / 2) / kSplitElems * kSplitElems;
            while (remaining > 0) {
                const int64_t take = remaining < per ? remaining : per;
                out->push_back(Piece{chunk, s.slot, s.dtype, false, false, s.host + eoff * isz, eoff, take,
                                     take * isz, -1});
                used = true;
                remaining -= take;
                eoff += take;
            }
            continue;
        }
        while (remaining > 0) {
            const size_t off = align_up(fill, kSlotAlign);
            const int64_t space = off < cap ? (int64_t)(cap - off) : 0;
            const int64_t fit = space / isz;
            int64_t take = fit >= remaining ? remaining : fit / kSplitElems * kSplitElems;
            if (take == 0 || (staged && nseg == max_segments_per_chunk)) {
                if (used) ++chunk;
                fill = 0;
                nseg = 0;
                used = false;
                continue;
            }
            out->push_back(Piece{chunk, s.slot, s.dtype, gathered, staged, s.host + eoff * isz, eoff, take,
                                 take * isz, (int64_t)off});
            used = true;
            fill = off + (size_t)(take * isz);
            if (staged) ++nseg;
            remaining -= take;
            eoff += take;
        }
    }
}

// ---------------------------------------------------------------------------------------
// launch plan of a LoRA read-modify-write group
// ---------------------------------------------------------------------------------------
TuningKnobs tuning_knobs() {
    TuningKnobs k = {-1, -1, -1, -1, -1, -1, -1, -1, 0, {0, 0, 0, 0, 0, 0, 0, 0}, -1};
#ifdef TIDAL_TUNING_KNOBS
    auto read = [](const char* name, int lo, int hi) {
        const char* e = getenv(name);
        if (!e || !*e) return -1;
        const int v = atoi(e);
        return (v >= lo && v <= hi) ? v : -1;
    };
    k.mfma_rc = read("TIDAL_MFMA_RC", 1, 1024);
    k.mfma_lds = read("TIDAL_MFMA_LDS", 0, 1);
    k.mfma_pair = read("TIDAL_MFMA_PAIR", 0, 1);
    k.mfma_order = read("TIDAL_MFMA_ORDER", 0, 3);
    k.mfma_dynlds = read("TIDAL_MFMA_DYNLDS", 0, 120 << 10);
    k.apply_ct = read("TIDAL_APPLY_CT", 1, kApplyChunkTiles);
    k.apply_tile_rows = read("TIDAL_APPLY_TILE_ROWS", 16, 32);
    if (k.apply_tile_rows != 16 && k.apply_tile_rows != 32) k.apply_tile_rows = -1;
    k.trace_host = read("TIDAL_TRACE_HOST", 0, 1);
    if (const char* e = getenv("TIDAL_UP_GROUPS")) {
        while (*e && k.n_up_groups < 8) {
            char* end = nullptr;
            const long cnt = strtol(e, &end, 10);
            if (end == e || cnt <= 0) break;
            k.up_groups[k.n_up_groups++] = (int)cnt;
            e = *end == ',' ? end + 1 : end;
        }
    }
    k.apply_two_step = read("TIDAL_APPLY_TWO_STEP", 0, 1);
#endif
    return k;
}

LoraLaunchPlan plan_lora_launch(const LoraGroup& g, bool ordered) {
    LoraLaunchPlan p = {};
    p.kind = kLoraNone;
    p.ks_old = g.rp_old / 16;
    p.ks_new = g.rp_new / 16;
    p.fork = g.fork;
    if (g.n_targets <= 0 || g.out <= 0 || g.in <= 0 || p.ks_old + p.ks_new == 0) return p;
    if (ordered) {
        p.kind = kLoraOrdered;
        p.waves_per_simd = 1;
        p.strips = (g.in + 255) / 256;                     // 64 x 256 tiles
        p.rowblocks = (g.out + 63) / 64;
        p.rc = 1;
        p.blocks_per_target = p.strips * p.rowblocks;
        p.total_blocks = (int64_t)p.blocks_per_target * g.n_targets;
        return p;
    }
    const TuningKnobs knobs = tuning_knobs();
    const int ks0 = p.ks_old, ks1 = p.ks_new;
    // A strips stay in registers except in swaps with a 64-rank side: there they are staged in LDS
    // (measured on 128 x 4096^2, LDS against registers: 64 -> 64 6.4 against 5.9 TB/s, 16/32 -> 64 6.5
    // against 6.1-6.25, 64 -> 16/32 6.5 against 6.1-6.2; merges of 64 ranks run at 6.5 either way).
    bool lds = !g.fork && ks0 > 0 && ks1 > 0 && (ks0 == 4 || ks1 == 4);
    if (knobs.mfma_lds >= 0) lds = knobs.mfma_lds != 0;
    lds = lds && !g.fork && lds_kernel_exists(ks0, ks1);
    // Tiles two at a time (32 live accumulator registers instead of 128) for every swap and for
    // 64-rank merges; merges of 16 or 32 ranks are faster with all tiles live.
    p.pair = (ks0 > 0 && ks1 > 0) || ks0 + ks1 >= 4;
    if (knobs.mfma_pair >= 0) p.pair = knobs.mfma_pair != 0;
    p.strips = (g.in + 255) / 256;
    p.rowblocks = (g.out + 31) / 32;
    const int64_t tiles = (int64_t)p.strips * p.rowblocks * g.n_targets;
    const bool pow2_pitch = (g.in & (g.in - 1)) == 0;
    // 32-row blocks per wave.  Short walks keep waves short-lived, which this memory system rewards,
    // long walks amortise the A strip, which grows with the rank; small jobs get fewer so that every
    // CU has work.  Measured per instantiation on 64 and 128 x 4096^2, 40 x 5120^2 and 15 of the two
    // 13824-wide shapes.
    int rc;
    if (lds) {
        p.kind = kLoraMfmaLds;
        p.pair = ks0 + ks1 < 8;          // 64 -> 64 is 2 % faster with all eight tiles live
        p.waves_per_simd = 1;            // the compiler fits two (64 -> 64 and 16/32 -> 64) or three (64 -> 16/32)
        // 16 for 64 -> 64, else 8; 4 and 2 where the row pitch is no power of two
        rc = (ks0 + ks1 >= 8) ? (pow2_pitch ? 16 : 4) : (pow2_pitch ? 8 : 2);
    } else {
        p.kind = kLoraMfmaReg;
        p.waves_per_simd = (p.pair && two_waves_fit(ks0, ks1)) ? 2 : 1;
        if (p.pair) {
            // swaps where two waves share a SIMD want 4 blocks, a 64-rank merge 8, every other swap
            // 16; on row pitches that are no power of two the short walks gain more: the 4 and the 8
            // are halved.  (A 16-rank merge looks 2-3 % faster at 2 blocks in a sweep where all slots
            // share one adapter; with an adapter per slot, as in the 70B-shaped stack, it is 1 %
            // slower: the A strips then come from HBM, not from L2.)
            rc = two_waves_fit(ks0, ks1) ? 4 : ((ks0 == 0 || ks1 == 0) ? 8 : 16);
            if (!pow2_pitch && rc <= 8) rc /= 2;
        } else {
            // merges of up to 32 ranks, all tiles live: 4 blocks on the 8-KB row pitch of 4096-wide
            // matrices (84 % of HBM peak against 82 % at 2), 2 on every other pitch measured -- 5120,
            // 8192, 11008, 28672 wide: 1 to 3 points more than at 4 (the A strip, once its loads were one
            // contiguous kilobyte each, stopped being what a short walk pays for)
            rc = 2 * g.in <= 8192 ? 4 : 2;
        }
    }
    const int64_t by_size = tiles / 4096;
    if (by_size < rc) rc = by_size < 1 ? 1 : (int)by_size;
    if (knobs.mfma_rc >= 1) rc = knobs.mfma_rc;
    p.rc = rc;
    if (lds) {
        const int rowchunks = (p.rowblocks + 4 * rc - 1) / (4 * rc);      // the four waves interleave 4*rc blocks
        p.blocks_per_target = p.strips * rowchunks;
    } else {
        const int rowchunks = (p.rowblocks + rc - 1) / rc;
        p.blocks_per_target = (p.strips * rowchunks + 3) / 4;             // one (strip, row chunk) per wave
    }
    p.total_blocks = (int64_t)p.blocks_per_target * g.n_targets;
    return p;
}

}  // namespace tidal
