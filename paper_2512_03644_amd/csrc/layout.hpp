// Host-side layout of a snapshot: validation of the segment list, stream offsets, parameter
// groups, tiling.  No GPU calls in here.
#pragma once
#include <stdint.h>

#include <vector>

#include "../../include/ffsnap.h"

namespace ffsnap {

struct Seg {
    uint64_t ptr;     // device address
    uint64_t off;     // stream offset of the first byte
    uint64_t nbytes;  // > 0
    uint32_t dtype, kind, param_id;
};

struct Param {
    uint32_t param_id;
    int32_t seg[4];   // indices into Layout::segs for W16, MASTER, M, V (-1 = missing)
    uint64_t numel;
};

struct Layout {
    uint64_t chunk_bytes = 0, payload = 0, n_chunks = 0, buffer_bytes = 0;
    std::vector<Seg> segs;      // non-empty segments, stream order
    std::vector<Param> params;  // ascending param_id
    bool adam_ok = false;       // every non-RAW segment belongs to a complete, consistent group
    uint32_t layout_id = 0;
    // tiling: a tile is the stream range one wavefront folds; it never crosses a chunk
    uint64_t tile_bytes = 0, n_tiles = 0;
    uint32_t tiles_per_chunk = 0;
    std::vector<uint32_t> tile_first_seg;  // segment holding the first byte of each tile
                                           // (segs.size()-1 for tiles past the payload)
};

// Returns FF_OK or a negative ff_status; `out` is valid only on FF_OK.
// tile_log2: 0 = default tile size, else log2 of the tile size in bytes (clamped to
// [10, log2(chunk_bytes)]).
int build_layout(const ff_segment* segs, uint64_t n_segs, uint64_t chunk_bytes, unsigned tile_log2,
                 Layout& out);

constexpr uint64_t kDefaultTileBytes = 1ull << 20;

}  // namespace ffsnap
