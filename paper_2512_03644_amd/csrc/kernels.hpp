// Launch wrappers of the GPU kernels (kernels.hip).  Every wrapper enqueues on `stream`,
// returns hipSuccess or the launch error, and never synchronises.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "xcd_order.h"

namespace ffsnap {

// Run length of the XCD-aware workgroup order (xcd_order.h) of the kernels that move 32 KiB per
// wavefront, 128 KiB per workgroup.
constexpr uint32_t kDefaultXcdGroup = 2048;

// Device-side view of a plan's tables, plus the constants the tile kernels need.
struct TileTables {
    const uint64_t* seg_off = nullptr;        // [n_seg + 1] stream offsets, seg_off[n_seg] = payload
    const uint64_t* seg_ptr = nullptr;        // [n_seg] device addresses
    const uint32_t* tile_first_seg = nullptr; // [n_tiles]
    const uint64_t* tile_base = nullptr;      // [n_tiles] tensor-side address of a tile that lies
                                              // inside one segment, else 0 (may be absent)
    const uint32_t* tab_u = nullptr;          // [4][256] multiply-by-x^8192 byte tables, then
                                              // [64] lane constants x^(128 * (63 - lane))
    // Where a tile's register goes.  acc set: XORed (atomically) into acc[chunk of the tile], an
    // array of the caller that launch_preset has prepared; nothing else is written, so calls that
    // share these tables may overlap in time.  Else partial set: stored to partial[tile] (a
    // buffer CRC over caller-provided scratch).  Neither: the pass only moves bytes.
    uint32_t* acc = nullptr;
    uint32_t* partial = nullptr;
    // If set: [plan tiles per chunk] x^(32 + 8 * bytes from the end of tile k of a chunk to the
    // end of the chunk).  A tile's register, which lacks the factor x^32 of a CRC register, is
    // multiplied by its entry, so that the registers of a chunk combine by XOR alone.  A pass
    // that folds groups of shift_stride plan tiles as one uses the entry of the group's last tile.
    const uint32_t* tile_shift = nullptr;
    uint32_t shift_stride = 1;
    uint64_t payload = 0;                     // N
    uint64_t total_rows = 0;                  // 1 KiB rows in the buffer
    uint32_t n_seg = 0;
    uint32_t tile_rows = 0;                   // rows per tile
    uint32_t lead_rows = 0;                   // rows missing at the front of tile 0
    uint32_t n_tiles = 0;
    uint32_t hint = 3;                        // bit 0: non-temporal tensor-side accesses, bit 1: buffer-side
    uint32_t n_list = 0;                      // > 0 selects tiles [tile_begin, tile_begin + n_list)
    uint32_t tile_begin = 0;
    const uint32_t* skip_bad = nullptr;       // if set: bad[] per chunk; tiles of bad chunks are left out
    uint32_t tiles_per_chunk = 1;             // of this pass (a power of two) ...
    uint32_t tpc_log2 = 0;                    // ... and its logarithm
    // Workgroups are dealt to the 8 XCDs round-robin.  With xcd_group = G > 0 the workgroups of
    // one XCD take G consecutive groups of tiles, the next XCD the following G, and so on, so
    // that every XCD (and its L2) sweeps runs of G * 128 KiB instead of every eighth 128 KiB.
    uint32_t xcd_group = kDefaultXcdGroup;  // measured: 8 .. 2048 within 0.5 % on a 12 GB shard, 2048 best
                                // (by 1-2 %) on a 15 GB one; 0 (launch order) costs 5-7 %
};

enum TileMode { kPack = 0, kRestore = 1, kVerify = 2 };

// A list of chunks handed to a kernel by value, inside its arguments: a selective restore needs
// no device memory of its own for it.  Longer lists are processed in several launches.
constexpr uint32_t kMaxListedChunks = 254;
struct ChunkList {
    uint32_t n = 0;
    uint32_t id[kMaxListedChunks];
};

// Folds every tile: kPack gathers segments -> chunks; kRestore reads chunks and scatters to the
// segments; kVerify only reads chunks.  With `list` (kRestore / kVerify, registers into t.acc)
// only the tiles of the listed chunks are processed.
hipError_t launch_tiles(TileMode mode, const TileTables& t, void* chunks, hipStream_t stream,
                        const ChunkList* list = nullptr);

// out[j] = affine (crcs null: pack) or affine ^ crcs[j] (verify) for chunks [first, first + n), or
// for the listed chunks; *n_bad = 0 if n_bad is not null.  The tiles then XOR their registers in.
hipError_t launch_preset(uint32_t* out, const uint32_t* crcs, uint64_t first, uint64_t n,
                         uint32_t affine, uint64_t* n_bad, const ChunkList* list,
                         hipStream_t stream);

// bad[j] = (bad[j] != 0) for chunks [0, n), or for the listed chunks; *n_bad += their number.
hipError_t launch_finish_verify(uint32_t* bad, uint64_t n, uint64_t* n_bad, const ChunkList* list,
                                hipStream_t stream);

// CRC of one buffer: combine n_tiles registers, then run the register over `tail_bytes` more
// bytes at `tail`, then apply the preset/complement term `affine`.
hipError_t launch_finish_crc(const uint32_t* partial, uint32_t n_tiles, uint32_t x_tile,
                             const uint8_t* tail, uint32_t tail_bytes, uint32_t affine,
                             uint32_t* out, hipStream_t stream);

// Verify pass over every chunk of a buffer with one workgroup per chunk (no atomics on the
// per-chunk words, no preset, no finish): sets *n_bad = 0, then bad[j] and *n_bad.  Usable when
// verify_chunks_applicable(); t supplies the tables (tile_shift for the plan's own tile size).
bool verify_chunks_applicable(uint64_t chunk_bytes, uint64_t n_chunks);
hipError_t launch_verify_chunks(const TileTables& t, uint64_t chunk_bytes, uint32_t tile_bytes,
                                uint32_t plan_tiles_per_chunk, uint32_t affine, const void* chunks,
                                const uint32_t* crcs, uint32_t* bad, uint64_t* n_bad,
                                uint64_t n_chunks, hipStream_t stream);

hipError_t launch_zero_u64(uint64_t* p, hipStream_t stream);

hipError_t launch_copy(void* dst, const void* src, uint64_t nbytes, hipStream_t stream);

// Fills tab (host, kTabWords entries): byte tables of multiplication by x^8192, then the 64 lane
// constants x^(128 * (63 - lane)).
constexpr int kTabWords = 1024 + 64;
void build_tab_u(uint32_t* tab);

}  // namespace ffsnap
