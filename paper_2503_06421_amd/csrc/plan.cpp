// Host-only planning for libtidal: configuration defaults, arena layout, copy plan.
#include "plan.h"

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
    }
    if (c.chunk_bytes == 0) c.chunk_bytes = (size_t)128 << 20;
    if (c.max_rank == 0) c.max_rank = 64;
    if (c.coalesce_bytes == 0) c.coalesce_bytes = (size_t)64 << 10;
    if (c.gather_threads == 0) c.gather_threads = 4;
    c.chunk_bytes = align_up(c.chunk_bytes, 4096);
    c.max_adapter_bytes = align_up(c.max_adapter_bytes, kSlotAlign);
    if (c.chunk_bytes < ((size_t)64 << 10)) { *msg = "chunk_bytes below 64 KiB"; return false; }
    if (c.chunk_bytes > ((size_t)1 << 32)) { *msg = "chunk_bytes above 4 GiB"; return false; }
    if (c.max_rank < 0 || c.max_rank > 64) { *msg = "max_rank outside 1..64"; return false; }
    if (c.coalesce_bytes > c.chunk_bytes) { *msg = "coalesce_bytes above chunk_bytes"; return false; }
    if (c.gather_threads < 1 || c.gather_threads > 16) { *msg = "gather_threads outside 1..16"; return false; }
    const int32_t known = TIDAL_FLAG_ORDERED_ACCUM | TIDAL_FLAG_TWO_PASS_SWAP | TIDAL_FLAG_SLOT_EVENTS |
                          TIDAL_FLAG_KERNEL_TIMING | TIDAL_FLAG_ASYNC_ENQUEUE | TIDAL_FLAG_NO_COPY_MERGE |
                          TIDAL_FLAG_PIPELINED_UPLOAD;
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

}  // namespace tidal
