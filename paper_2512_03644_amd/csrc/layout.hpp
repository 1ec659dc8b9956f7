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
    uint32_t half_dtype = 0;    // format of the working weights: FF_BF16 or FF_F16 (0: no groups)
    uint32_t layout_id = 0;
    // tiling: a tile is the stream range one wavefront folds; it never crosses a chunk
    uint64_t tile_bytes = 0, n_tiles = 0;
    uint32_t tiles_per_chunk = 0;
    std::vector<uint32_t> tile_first_seg;  // segment holding the first byte of each tile
                                           // (segs.size()-1 for tiles past the payload)
    // Tensor-side address of a tile's first byte if the whole tile lies inside one segment, else
    // 0: lets a wavefront start such a tile after one table read instead of a walk through the
    // segment tables.
    std::vector<uint64_t> tile_base;
};

// Unit of work of the fused optimizer step: a run of elements of one parameter group (its four
// streams w16/master/m/v), or a run of bytes of a RAW segment.  Runs are cut wherever one of
// their streams crosses a chunk boundary, so each stream of a tile lies inside one chunk and
// adds one term ("piece") to that chunk's CRC: register(piece) * x^(8 * bytes from the end of
// the piece to the end of the chunk).  An fp32 element that straddles a chunk boundary (its
// stream offset is 2 mod 4) starts a tile; its first two bytes form a separate "head" piece
// that ends the previous chunk.
struct WorkTile {
    uint64_t ptr[4];    // addresses of the tile's first element: w16, master, m, v (RAW: ptr[0])
    uint64_t soff[4];   // stream offsets of the tile's first byte in each stream
    uint32_t chunk[7];  // pieces 0..3: the four streams; 4..6: head pieces of master, m, v
    uint32_t shift[7];  // x^(8 * distance to the chunk end) mod P; 0 = piece absent
    uint64_t e0;        // first element within the parameter (indexes the gradient)
    uint32_t n;         // elements (parameter tile) or bytes (RAW tile)
    uint32_t kind;      // 0 = parameter group, 1 = RAW
    uint32_t grad_index;
    uint32_t head_split;  // bit x set: the first element of stream x is split as described
};

constexpr uint32_t kWorkParam = 0, kWorkRaw = 1;
constexpr uint32_t kParamTileElems = 1u << 13;
constexpr uint32_t kRawTileBytes = 1u << 15;

// Work list of the fused step over the whole layout (needs L.adam_ok): the parameter tiles first,
// then the RAW tiles.
void build_work_tiles(const Layout& L, std::vector<WorkTile>& out);

// Returns FF_OK or a negative ff_status; `out` is valid only on FF_OK.
// tile_log2: 0 = default tile size, else log2 of the tile size in bytes (clamped to
// [10, log2(chunk_bytes)]).
int build_layout(const ff_segment* segs, uint64_t n_segs, uint64_t chunk_bytes, unsigned tile_log2,
                 Layout& out);

// 32 KiB tiles keep the region the chip is sweeping at any moment compact, which is what a pass
// that reads and writes needs; a read-only pass amortises the per-tile reduction better on 64 KiB.
constexpr uint64_t kDefaultTileBytes = 1ull << 15;
constexpr uint64_t kVerifyTileBytes = 1ull << 16;

}  // namespace ffsnap
