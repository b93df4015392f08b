// Host-only planning: slot placement and the chunked copy plan of a materialisation.
// No HIP call is made here, so this part can be exercised without a GPU.
#ifndef TIDAL_PLAN_H_
#define TIDAL_PLAN_H_

#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "tidal.h"

namespace tidal {

constexpr size_t kSlotAlign = 256;        // every slot, staging piece and packed factor starts on this
constexpr int64_t kSplitElems = 128;      // tensors are split between chunks at multiples of this

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t dtype_size(int32_t d) { return d == TIDAL_F32 ? 4 : 2; }
inline bool dtype_ok(int32_t d) { return d == TIDAL_F32 || d == TIDAL_F16 || d == TIDAL_BF16; }

struct ArenaLayout {
    std::vector<size_t> slot_offset;   // n + 1 entries; last = size of the slot area
    size_t staging[2];
    size_t adapter_region[2];
    size_t total;
};

// Slot i holds rows*cols bf16 at a 256-byte aligned offset, in the order given (the traced
// access order of the paper's Sec. 4.2); then the library's own areas.
bool layout_arena(const tidal_slot_desc* slots, int32_t n, const tidal_config& cfg, ArenaLayout* out);

// Fill defaults and validate.  Returns false (with msg) when a field is out of range.
bool normalise_config(const tidal_config* in, tidal_config* out, const char** msg);

struct Piece {
    int32_t chunk;
    int32_t slot;
    int32_t dtype;
    bool gathered;          // goes through the CPU-filled pinned buffer of its chunk
    bool staged;            // lands in the device staging buffer and is converted from there
    const char* host;       // first source byte of the piece
    int64_t elem_offset;    // within the slot
    int64_t elems;
    int64_t src_bytes;
    int64_t buf_offset;     // byte offset inside the chunk's pinned / staging buffer; -1 = unused
};

struct SourceInfo {
    int32_t slot;
    int32_t dtype;
    const char* host;
    int64_t elems;
    bool pinned;
};

// Cut the sources, in order, into copy pieces grouped in chunks of at most chunk_bytes of
// buffer space (the paper's Sec. 6: fewer, larger copies instead of one per tensor; here
// also: large tensors split so that copy and conversion of successive chunks overlap).
void plan_copies(const std::vector<SourceInfo>& srcs, const tidal_config& cfg, int max_segments_per_chunk,
                 std::vector<Piece>* out);

}  // namespace tidal
#endif
