// GPU kernels of the snapshot path for gfx950 (CDNA4, 64-wide wavefronts).
//
// Layout of the work.  The chunk buffer is cut into tiles (a power-of-two number of 1 KiB rows,
// never crossing a chunk).  One wavefront owns one tile and walks it row by row; in a row lane l
// handles the 16 bytes at offset 16*l, so every global access of the wavefront is one
// contiguous, 16-byte-per-lane, 1 KiB transaction on the buffer side.  On the tensor side the
// same 16 bytes come from (pack) or go to (restore) wherever the stream position falls in the
// segment list: a row that lies inside one segment is a single, possibly unaligned, 16-byte
// access per lane; a row that touches a segment boundary is assembled halfword by halfword.
//
// CRC32C without table lookups in the inner loop.  A lane sees 4 dwords per row, 256 dwords
// apart from row to row.  It keeps NE*4 dwords of state that represent its part of the message
// as a polynomial in y = x^32; every row multiplies the state by y^256 (a rotation of register
// names) and the 4 dwords that leave the top are XORed into 9 tap positions each, using sparse
// multiples of the CRC generator (fold_taps.h).  That is 36 XORs per 16 bytes and is exact
// GF(2) algebra.  Only at the end of a tile are the NE*4 dwords of every lane reduced to one
// 32-bit register: Horner steps with byte tables (multiply by x^8192) held in LDS, then
// bitwise multiplications to merge columns and lanes.  The tile multiplies that register by
// x^(8 * bytes between its end and the end of its chunk) and XORs it, with an atomic, into the
// chunk's word of the caller's own output array (crcs[] for pack, bad[] for restore/verify), which
// a small kernel has preset with the preset/complement term of the CRC.  XOR commutes, so the
// result does not depend on the order in which tiles finish, and no memory outside the caller's
// arrays is written: calls on one plan may overlap in time.
#include "kernels.hpp"

#include "fold.h"

namespace ffsnap {

namespace {

constexpr int kWavesPerBlock = 4;
using Fold = Fold16x16;
constexpr int kRowBytes = Fold::ROW_BYTES;
constexpr int kNE = Fold::NE;
constexpr int kNF = Fold::NF;
// rows in flight per wavefront on the general path (restore keeps fewer: its general path is the
// point of highest register pressure of the kernel, and four more rows there would push the whole
// kernel past the 256 registers that two wavefronts per SIMD allow)
template <int MODE>
constexpr int kDepthOf = (MODE == kRestore) ? 4 : 8;
// A default-size tile that lies inside one segment is processed by straight-line code with a
// deeper queue: with no loop there is no loop-carried register to copy and no wait for all
// outstanding loads at a loop head.
constexpr int kWholeRows = 32;   // rows of a default (32 KiB) tile
constexpr int kRealignDepth = 16;  // rows in flight on the restore path that re-aligns its stores
constexpr int kRingWords = 520;  // two rows and 16 bytes, as dwords, padded to a multiple of 16 bytes
constexpr int kVerifyRows = 64;  // a read-only pass walks its grouped tile in blocks of 64 rows
// rows requested before the first store on that path (measured on the 7B and 70B/64 shards: with
// the stores going to the chunk buffer 26-30 rows are best, 1 % ahead of 16 and of the whole
// tile; with the stores going to the tensors the whole tile is; a read-only pass keeps 16)
template <int MODE>
constexpr int kWholeDepth = (MODE == kRestore) ? 32 : (MODE == kPack) ? 28 : 16;
static_assert(kNE % kDepthOf<kPack> == 0 && kNE % kDepthOf<kRestore> == 0,
              "queue slots must repeat with the state rotation");
static_assert(kNF == 4 && kRowBytes == 1024, "one 16-byte word per lane per row");

// ---- segment cursor (wave-uniform) -----------------------------------------------------------

struct Cursor {
    uint32_t si;    // current segment
    uint64_t a, b;  // its stream range [a, b)
    uint64_t base;  // its device address
};

__device__ __forceinline__ void cursor_init(Cursor& c, const uint64_t* __restrict__ seg_off,
                                            const uint64_t* __restrict__ seg_ptr, uint32_t si)
{
    c.si = si;
    c.a = seg_off[si];
    c.b = seg_off[si + 1];
    c.base = seg_ptr[si];
}

// Move to the segment that holds stream offset s (the last segment if s is past the payload).
__device__ __forceinline__ void cursor_seek(Cursor& c, const uint64_t* __restrict__ seg_off,
                                            const uint64_t* __restrict__ seg_ptr, uint32_t n_seg,
                                            uint64_t s)
{
    bool moved = false;
    while (s >= c.b && c.si + 1 < n_seg) {
        c.si++;
        c.a = c.b;
        c.b = seg_off[c.si + 1];
        moved = true;
    }
    while (s < c.a) {
        c.si--;
        c.b = c.a;
        c.a = seg_off[c.si];
        moved = true;
    }
    if (moved) c.base = seg_ptr[c.si];
}

// Per-lane: index of the segment holding stream offset pos, searching upwards from si0, the
// segment that holds the start of the lane's row.  The answer is nearly always si0 or its
// successor, so the search gallops (steps of 1, 2, 4, ...) until it has passed pos and then
// bisects the last step: one table read when the answer is si0, three when it is si0 + 1.
__device__ __forceinline__ uint32_t find_segment(const uint64_t* __restrict__ seg_off,
                                                 uint32_t n_seg, uint32_t si0, uint64_t pos)
{
    uint32_t lo = si0, step = 1;
    while (lo + step < n_seg && seg_off[lo + step] <= pos) {
        lo += step;
        step <<= 1;
    }
    // seg_off[lo] <= pos, and seg_off[lo + step] > pos or lo + step is past the last segment
    uint32_t hi = (lo + step < n_seg) ? lo + step - 1 : n_seg - 1;
    while (lo < hi) {
        const uint32_t mid = lo + (hi - lo + 1) / 2;
        if (seg_off[mid] <= pos)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// A row that is not wholly inside one segment: every lane finds its own 16 bytes.
__device__ __noinline__ u32x4 gather_row_slow(const uint64_t* __restrict__ seg_off,
                                              const uint64_t* __restrict__ seg_ptr, uint32_t n_seg,
                                              uint32_t si0, uint64_t s, uint64_t payload, int lane)
{
    const uint64_t pos = s + 16u * lane;
    uint32_t j = find_segment(seg_off, n_seg, si0, pos);
    uint64_t a = seg_off[j], b = seg_off[j + 1], base = seg_ptr[j];
    if (pos + 16 <= b) return load16_unaligned(reinterpret_cast<const uint8_t*>(base + (pos - a)));
    uint32_t h[8];
#pragma unroll
    for (int u = 0; u < 8; u++) {
        const uint64_t p = pos + 2u * u;
        while (p >= b && j + 1 < n_seg) {
            j++;
            a = b;
            b = seg_off[j + 1];
            base = seg_ptr[j];
        }
        h[u] = (p < payload) ? *as_global(reinterpret_cast<const uint16_t*>(base + (p - a))) : 0u;
    }
    u32x4 r;
    r.x = h[0] | (h[1] << 16);
    r.y = h[2] | (h[3] << 16);
    r.z = h[4] | (h[5] << 16);
    r.w = h[6] | (h[7] << 16);
    return r;
}

__device__ __noinline__ void scatter_row_slow(const uint64_t* __restrict__ seg_off,
                                              const uint64_t* __restrict__ seg_ptr, uint32_t n_seg,
                                              uint32_t si0, uint64_t s, uint64_t payload, int lane,
                                              u32x4 w)
{
    const uint64_t pos = s + 16u * lane;
    uint32_t j = find_segment(seg_off, n_seg, si0, pos);
    uint64_t a = seg_off[j], b = seg_off[j + 1], base = seg_ptr[j];
    if (pos + 16 <= b) {
        store16_unaligned(reinterpret_cast<uint8_t*>(base + (pos - a)), w);
        return;
    }
    const uint32_t d[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int u = 0; u < 8; u++) {
        const uint64_t p = pos + 2u * u;
        while (p >= b && j + 1 < n_seg) {
            j++;
            a = b;
            b = seg_off[j + 1];
            base = seg_ptr[j];
        }
        if (p < payload)
            *as_global(reinterpret_cast<uint16_t*>(base + (p - a))) =
                static_cast<uint16_t>(d[u >> 1] >> ((u & 1) * 16));
    }
}

template <int J>
__device__ __forceinline__ void fold_word(uint32_t (&S)[kNE][kNF], u32x4 w)
{
    const uint32_t d[4] = {w.x, w.y, w.z, w.w};
    fold_row<Fold, J>(S, d);
}

// ---- tile kernel -------------------------------------------------------------------------------

// Three bodies, fastest first.  (1) A default-size tile that lies inside one segment (and a
// read-only tile of the grouped size) is one piece of straight-line code over all its rows; on
// restore, such a tile whose place in the tensor is off the 128-byte lines takes a variant that
// lines its stores up through LDS.
// (2) A default-size tile that touches up to four segments or the end of the payload is
// straight-line too, every lane choosing its segment by comparisons.  (3) Everything else -- other
// tile sizes, many small segments, tiles behind the payload -- walks its rows in groups of kNE (one
// full rotation of the state registers): a group whose rows, and the rows it prefetches, all lie
// inside one segment runs without branches between its loads, kDepth of them in flight; any other
// group (virtual rows at the tile start, a segment boundary, the end of the payload) takes the
// guarded path row by row.
template <int MODE, int HINT>
__device__ __forceinline__ void tile_body(
    const uint64_t* __restrict__ seg_off, const uint64_t* __restrict__ seg_ptr,
    const uint32_t* __restrict__ tile_first_seg, const uint32_t* __restrict__ tab_u_global,
    uint32_t* __restrict__ partial, uint32_t* __restrict__ acc, uint8_t* __restrict__ chunks,
    const TileTables& T, const uint32_t* tab, uint32_t* ring, const uint32_t tile, const int lane)
{
    // constant that moves this tile's register to the end of its chunk (tiles per chunk is a
    // power of two) and supplies the factor x^32 the register lacks; fetched now, used after the
    // last row
    const uint32_t shift =
        T.tile_shift ? T.tile_shift[((tile & (T.tiles_per_chunk - 1)) + 1) * T.shift_stride - 1] : 0u;
    auto store_register = [&](uint32_t reg) {
        if (T.tile_shift) reg = gf2_mul(reg, shift);
        if (lane == 0) {
            if (acc)
                atomicXor(acc + (tile >> T.tpc_log2), reg);
            else
                partial[tile] = reg;
        }
    };
    // a pass that only moves bytes (the scatter pass behind a verify pass) folds nothing
    const bool folding = (acc != nullptr) || (partial != nullptr);

    // rows of this tile, as indices into the buffer's rows
    const int64_t g0 = static_cast<int64_t>(tile) * T.tile_rows - T.lead_rows;
    const int64_t row_begin = g0 < 0 ? 0 : g0;
    const int R = static_cast<int>(g0 + T.tile_rows - row_begin);
    const int groups = (R + kNE - 1) / kNE;
    const int pad = groups * kNE - R;  // virtual zero rows in front: they leave the state at 0
    const uint64_t s_base = static_cast<uint64_t>(row_begin) * kRowBytes;
    const uint32_t lane16 = 16u * lane;
    constexpr bool kSegNT = (HINT & 1) != 0;  // non-temporal accesses on the tensor side
    constexpr bool kBufNT = (HINT & 2) != 0;  // non-temporal accesses on the chunk-buffer side

    uint32_t S[kNE][kNF];
    static_for<kNE>([&](auto e) { static_for<kNF>([&](auto f) { S[e][f] = 0; }); });

    // Whole-tile paths: all rows real and, on the tensor side, inside one segment.
    auto whole_rows = [&](auto rows_c, auto depth_c, const uint8_t* bp, const uint8_t* tp) {
        constexpr int kRows = rows_c, kD = depth_c;
        static_assert(kRows % kNE == 0 && kD <= kRows, "whole-tile path");
        auto fetch = [&](int r) {
            return (MODE == kPack) ? load16_unaligned<kSegNT>(tp + r * kRowBytes)
                                   : load16_stream<kBufNT>(bp + r * kRowBytes);
        };
        u32x4 w[kD];
        static_for<kD>([&](auto k) { w[k] = fetch(k); });
        static_for<kRows>([&](auto Jc) {
            constexpr int J = Jc;
            const u32x4 x = w[J % kD];
            if (MODE == kPack) store16_stream<kBufNT>(const_cast<uint8_t*>(bp) + J * kRowBytes, x);
            if (MODE == kRestore)
                store16_unaligned<kSegNT>(const_cast<uint8_t*>(tp) + J * kRowBytes, x);
            fold_word<J % kNE>(S, x);
            if constexpr (J + kD < kRows) {
                __builtin_amdgcn_sched_barrier(0);
                w[J % kD] = fetch(J + kD);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };
    auto whole_tile = [&](auto rows_c, auto depth_c, const uint8_t* bp, const uint8_t* tp) {
        whole_rows(rows_c, depth_c, bp, tp);
        if (folding) store_register(reduce_state<Fold>(S, tab, tab_u_global[1024 + lane]));
    };
    // Restore of a whole tile whose place in its tensor does not start on a 128-byte line.  Stored
    // as loaded, every row would be a 1 KiB store that straddles line boundaries at both ends and
    // in every 256-byte quarter.  Instead the rows pass through a two-row ring in LDS that belongs
    // to this wavefront alone and leave it shifted by the misalignment m: output row R holds the
    // tile's bytes [1024 R - m, 1024 R - m + 1024) and goes to a line-aligned address.  Rows 0 and
    // kWholeRows of the output are partial (the first lacks its leading m bytes, the last holds
    // only m) and are stored lane by lane, the lane on the edge halfword by halfword.  The fold
    // takes the rows as loaded, so the CRC is untouched.  LDS operations of one wavefront complete
    // in order, so a row written is visible to the reads that follow without a barrier.
    auto whole_tile_realigned = [&](const uint8_t* bp, const uint64_t t0) {
        constexpr int kRows = kWholeRows;
        const uint32_t m = static_cast<uint32_t>(t0) & 127u;
        uint8_t* const ap = reinterpret_cast<uint8_t*>(t0 - m) + lane16;  // lane's slot, output row 0
        // ring: rows at byte 1024 * (row & 1); bytes [2048, 2064) repeat bytes [0, 16) so that a
        // read that starts in the last 14 bytes runs on into the even row's beginning
        const uint32_t o0 = (lane16 - m) & 2047u;  // lane's first byte, even output rows
        const uint32_t o1 = (o0 + 1024u) & 2047u;  // odd output rows
        const uint32_t sh = (m & 2u) * 8u;         // the lane's bytes start this far into a dword
        const uint32_t* const r0 = ring + (o0 >> 2);
        const uint32_t* const r1 = ring + (o1 >> 2);
        auto take = [&](const uint32_t* r) {
            uint32_t d[5];
            static_for<5>([&](auto k) { d[k] = r[k]; });
            return u32x4{__builtin_amdgcn_alignbit(d[1], d[0], sh), __builtin_amdgcn_alignbit(d[2], d[1], sh),
                         __builtin_amdgcn_alignbit(d[3], d[2], sh), __builtin_amdgcn_alignbit(d[4], d[3], sh)};
        };
        // bytes [lo, hi) of an output row: whole slots as one store, the slot on an edge by halfwords
        auto store_part = [&](uint8_t* p, const u32x4 y, const uint32_t lo, const uint32_t hi) {
            if (lane16 >= lo && lane16 + 16u <= hi) {
                store16_stream<kSegNT>(p, y);
            } else if (lane16 + 16u > lo && lane16 < hi) {
                const uint32_t d[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
                for (int u = 0; u < 8; u++) {
                    const uint32_t pos = lane16 + 2u * u;
                    if (pos >= lo && pos < hi)
                        *as_global(reinterpret_cast<uint16_t*>(p + 2 * u)) =
                            static_cast<uint16_t>(d[u >> 1] >> ((u & 1) * 16));
                }
            }
        };
        constexpr int kD = kRealignDepth;
        u32x4 w[kD];
        static_for<kD>([&](auto k) { w[k] = load16_stream<kBufNT>(bp + k * kRowBytes); });
        static_for<kRows>([&](auto Jc) {
            constexpr int J = Jc;
            const u32x4 x = w[J % kD];
            *reinterpret_cast<u32x4*>(ring + (J & 1) * 256 + 4 * lane) = x;
            if ((J & 1) == 0 && lane == 0) *reinterpret_cast<u32x4*>(ring + 512) = x;
            const u32x4 y = take((J & 1) ? r1 : r0);
            fold_word<J % kNE>(S, x);
            if constexpr (J + kD < kRows) {
                __builtin_amdgcn_sched_barrier(0);
                w[J % kD] = load16_stream<kBufNT>(bp + (J + kD) * kRowBytes);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (J == 0)
                store_part(ap, y, m, kRowBytes);
            else
                store16_stream<kSegNT>(ap + J * kRowBytes, y);
        });
        store_part(ap + kRows * kRowBytes, take(r0), 0u, m);
        if (folding) store_register(reduce_state<Fold>(S, tab, tab_u_global[1024 + lane]));
    };
    // Pack: a default-size tile that the plan found inside one segment starts after a single
    // table read; the segment tables are walked only for the other tiles.  (Restore, whose loads
    // do not wait for a tensor address, measured 1 % slower that way and keeps the walk.)
    if (MODE == kPack && T.tile_base && T.tile_rows == kWholeRows &&
        R == static_cast<int>(T.tile_rows)) {
        const uint64_t tb = T.tile_base[tile];
        if (tb) {
            whole_tile(std::integral_constant<int, kWholeRows>{},
                       std::integral_constant<int, kWholeDepth<MODE>>{}, chunks + s_base + lane16,
                       reinterpret_cast<const uint8_t*>(tb) + lane16);
            return;
        }
    }

    Cursor cin, cout;  // pack reads through cin; restore writes through cout
    if (MODE == kPack) cursor_init(cin, seg_off, seg_ptr, tile_first_seg[tile]);
    if (MODE == kRestore) cursor_init(cout, seg_off, seg_ptr, tile_first_seg[tile]);

    auto row_offset = [&](int r) { return s_base + static_cast<uint64_t>(r) * kRowBytes; };

    // guarded single-row access
    auto load_row = [&](int r) -> u32x4 {
        const uint64_t s = row_offset(r);
        if (MODE == kPack) {
            if (s >= T.payload) return u32x4{0, 0, 0, 0};
            cursor_seek(cin, seg_off, seg_ptr, T.n_seg, s);
            if (s + kRowBytes <= cin.b)
                return load16_unaligned<kSegNT>(reinterpret_cast<const uint8_t*>(cin.base + (s - cin.a)) +
                                        lane16);
            return gather_row_slow(seg_off, seg_ptr, T.n_seg, cin.si, s, T.payload, lane);
        } else {
            return load16_stream<kBufNT>(chunks + s + lane16);
        }
    };
    auto sink_row = [&](int r, u32x4 w) {
        const uint64_t s = row_offset(r);
        if (MODE == kPack) {
            store16_stream<kBufNT>(chunks + s + lane16, w);
        } else if (MODE == kRestore) {
            if (s >= T.payload) return;
            cursor_seek(cout, seg_off, seg_ptr, T.n_seg, s);
            if (s + kRowBytes <= cout.b)
                store16_unaligned<kSegNT>(reinterpret_cast<uint8_t*>(cout.base + (s - cout.a)) + lane16, w);
            else
                scatter_row_slow(seg_off, seg_ptr, T.n_seg, cout.si, s, T.payload, lane, w);
        }
    };
    // Is the stream range [s, s + n rows) inside one segment?  On success *p is the lane's
    // address of the first row.  (Buffer-side ranges always are.)
    auto span_in_segment = [&](Cursor& c, uint64_t s, int n, const uint8_t** p) -> bool {
        if (s >= T.payload) return false;
        cursor_seek(c, seg_off, seg_ptr, T.n_seg, s);
        if (s + static_cast<uint64_t>(n) * kRowBytes > c.b) return false;
        *p = reinterpret_cast<const uint8_t*>(c.base + (s - c.a)) + lane16;
        return true;
    };

    if (R == static_cast<int>(T.tile_rows)) {
        const uint8_t* bp = chunks + s_base + lane16;  // buffer side
        const uint8_t* tp = bp;                        // tensor side
        if (MODE != kPack && T.tile_rows == kWholeRows) {
            bool whole = true;
            if (MODE == kRestore) whole = span_in_segment(cout, s_base, kWholeRows, &tp);
            if (whole) {
                if (MODE == kRestore && ring) {
                    const uint64_t t0 = cout.base + (s_base - cout.a);
                    if (t0 & 127u) {
                        whole_tile_realigned(bp, t0);
                        return;
                    }
                }
                whole_tile(std::integral_constant<int, kWholeRows>{},
                           std::integral_constant<int, kWholeDepth<MODE>>{}, bp, tp);
                return;
            }
        }
        if (MODE == kVerify && T.tile_rows % kVerifyRows == 0) {
            // a read-only pass folds a long tile as one message, block after block (a block is a
            // whole number of rotations of the state); one reduction and one atomic per tile
            const int blocks = static_cast<int>(T.tile_rows) / kVerifyRows;
            for (int blk = 0; blk < blocks; blk++) {
                whole_rows(std::integral_constant<int, kVerifyRows>{},
                           std::integral_constant<int, kWholeDepth<kVerify>>{}, bp, tp);
                bp += kVerifyRows * kRowBytes;
            }
            if (folding) store_register(reduce_state<Fold>(S, tab, tab_u_global[1024 + lane]));
            return;
        }
        // Piecewise path: a default-size tile that starts inside the payload and touches at most
        // kPieces segments; the end of the payload counts as one more boundary, behind which
        // lanes read zeros (pack) or store nothing (restore).  Every lane picks the segment of
        // its own 16 bytes by comparing its offset in the tile with the (wave-uniform) segment
        // boundaries, so a row that contains a boundary is still one vector access with per-lane
        // addresses and the code stays straight-line.  Only lanes whose 16 bytes straddle a
        // boundary cannot be served that way: they read a harmless address instead (their own
        // slot of the buffer row) and then move their 8 halfwords one by one, each located by
        // the same comparisons.
        if (MODE != kVerify && T.tile_rows == kWholeRows && s_base < T.payload) {
            constexpr int kPieces = 4;
            const uint32_t first = tile_first_seg[tile];
            static_assert(kPieces == 4, "the selection chains below are written out");
            // stream offsets of the first five segments from `first` on (seg_off[n_seg] is the
            // payload size); plain scalars throughout, so that everything stays in registers
            auto seg_begin = [&](uint32_t k) { return seg_off[first + k < T.n_seg ? first + k : T.n_seg]; };
            const uint64_t a0 = seg_begin(0), a1 = seg_begin(1), a2 = seg_begin(2), a3 = seg_begin(3),
                           a4 = seg_begin(4);
            if (a4 >= s_base + uint64_t(kWholeRows) * kRowBytes || a4 >= T.payload) {
                constexpr uint32_t kTileBytes = kWholeRows * kRowBytes;
                const uint64_t left = T.payload - s_base;  // payload bytes from the tile start on
                const uint32_t pend = left < kTileBytes ? static_cast<uint32_t>(left) : kTileBytes;
                // per segment, the address tile offset 0 would have if it lay in that segment
                // (modulo 2^64 for all but the first), and the boundaries relative to the tile
                // (>= kTileBytes: none)
                auto seg_base = [&](uint32_t k, uint64_t ak) {
                    return seg_ptr[first + k < T.n_seg ? first + k : T.n_seg - 1] + (s_base - ak);
                };
                auto rel_bound = [&](uint64_t ak) {  // ak > s_base
                    const uint64_t d = ak - s_base;
                    return d < kTileBytes ? static_cast<uint32_t>(d) : kTileBytes;
                };
                const uint64_t base0 = seg_base(0, a0), base1 = seg_base(1, a1), base2 = seg_base(2, a2),
                               base3 = seg_base(3, a3);
                const uint32_t rb0 = rel_bound(a1), rb1 = rel_bound(a2), rb2 = rel_bound(a3);
                // A lane's segment base is base0 plus the steps of the boundaries it lies behind.
                // (Sums of `condition ? step : 0` on purpose: a chain of `condition ? base_k : b`
                // over captured variables gets rewritten into a choice between their addresses
                // followed by a load, which forces them all into memory.)
                const uint64_t step1 = base1 - base0, step2 = base2 - base1, step3 = base3 - base2;
                auto lane_base = [&](uint32_t rel) {
                    return base0 + (rel >= rb0 ? step1 : 0) + (rel >= rb1 ? step2 : 0) +
                           (rel >= rb2 ? step3 : 0);
                };
                // per-lane address of the lane's 16 bytes of row J on the tensor side, whether
                // they straddle a boundary, and whether they lie wholly behind the payload
                auto locate = [&](int J, bool& straddle, bool& beyond) -> const uint8_t* {
                    const uint32_t rel = static_cast<uint32_t>(J) * kRowBytes + lane16;
                    beyond = rel >= pend;
                    straddle = (!beyond && rel + 16u > pend) || (rel < rb0 && rel + 16u > rb0) ||
                               (rel < rb1 && rel + 16u > rb1) || (rel < rb2 && rel + 16u > rb2);
                    return reinterpret_cast<const uint8_t*>(lane_base(rel) + rel);
                };
                // address of the halfword at tile offset rel2 (a halfword never straddles)
                auto locate_half = [&](uint32_t rel2) -> uint64_t { return lane_base(rel2) + rel2; };
                // Pack: the (at most kPieces) 16-byte slots of the tile that straddle a boundary
                // are fetched before anything else, halfword by halfword: lane 8k + u takes
                // halfword u of the slot that holds boundary k (k = kPieces - 1: the end of the
                // payload).  The owner of such a slot later collects its 8 halfwords from those
                // lanes, so no row of the tile has to wait for loads issued in that row.
                uint32_t fix = 0;
                if (MODE == kPack) {
                    const int k = lane >> 3, u = lane & 7;
                    const uint32_t bnd = pend + (k == 0 ? rb0 - pend : 0) + (k == 1 ? rb1 - pend : 0) +
                                         (k == 2 ? rb2 - pend : 0);
                    if (k < kPieces && bnd < kTileBytes && (bnd & 15u)) {
                        const uint32_t rel2 = (bnd & ~15u) + 2u * u;
                        if (rel2 < pend)
                            fix = *as_global(reinterpret_cast<const uint16_t*>(locate_half(rel2)));
                    }
                }
                // rows in flight: pack as on its whole-tile path; restore, whose stores here go to
                // per-lane addresses, does best with 16 (28: 3 % slower on tiles of two tensors)
                constexpr int kD = (MODE == kPack) ? kWholeDepth<kPack> : 16;
                auto fetch = [&](int J) -> u32x4 {
                    if (MODE == kRestore) return load16_stream<kBufNT>(bp + J * kRowBytes);
                    bool straddle, beyond;
                    const uint8_t* p = locate(J, straddle, beyond);
                    if (straddle || beyond) p = bp + J * kRowBytes;  // a valid address: value unused
                    return load16_unaligned<kSegNT>(p);
                };
                u32x4 w[kD];
                static_for<kD>([&](auto k) { w[k] = fetch(k); });
                static_for<kWholeRows>([&](auto Jc) {
                    constexpr int J = Jc;
                    u32x4 x = w[J % kD];
                    bool straddle, beyond;
                    const uint8_t* p = locate(J, straddle, beyond);
                    const uint32_t rel = static_cast<uint32_t>(J) * kRowBytes + lane16;
                    if (MODE == kPack) {
                        if (beyond) x = u32x4{0, 0, 0, 0};
                        static_for<kPieces>([&](auto kk) {
                            constexpr int k = kk;
                            const uint32_t bnd = k == 0 ? rb0 : k == 1 ? rb1 : k == 2 ? rb2 : pend;
                            if (bnd < kTileBytes && (bnd & 15u) && (bnd >> 10) == uint32_t(J)) {
                                uint32_t h[8];
                                static_for<8>([&](auto u) {
                                    h[u] = __builtin_amdgcn_readlane(fix, 8 * k + u);
                                });
                                if (uint32_t(lane) == ((bnd & 1023u) >> 4))
                                    x = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16),
                                              h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
                            }
                        });
                        store16_stream<kBufNT>(const_cast<uint8_t*>(bp) + J * kRowBytes, x);
                    } else {
                        if (straddle) {
                            const uint32_t d[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                            for (int u = 0; u < 8; u++) {
                                const uint32_t rel2 = rel + 2u * u;
                                if (rel2 < pend)
                                    *as_global(reinterpret_cast<uint16_t*>(locate_half(rel2))) =
                                        static_cast<uint16_t>(d[u >> 1] >> ((u & 1) * 16));
                            }
                        } else if (!beyond) {
                            store16_unaligned<kSegNT>(const_cast<uint8_t*>(p), x);
                        }
                    }
                    fold_word<J % kNE>(S, x);
                    // the fence also keeps the address arithmetic of later rows from being moved
                    // up here, where it would only hold registers
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (J + kD < kWholeRows) {
                        w[J % kD] = fetch(J + kD);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                });
                if (folding) store_register(reduce_state<Fold>(S, tab, tab_u_global[1024 + lane]));
                return;
            }
        }
    }

    // queue slot of row r is (r + pad) mod kDepth; fill the first kDepth rows
    constexpr int kDepth = kDepthOf<MODE>;
    u32x4 q[kDepth];
    {
        const uint8_t* lp = chunks + s_base + lane16;
        bool fast = (pad == 0) && (R >= kDepth);
        if (MODE == kPack) fast = fast && span_in_segment(cin, s_base, kDepth, &lp);
        if (fast) {
            static_for<kDepth>([&](auto k) {
                q[k] = (MODE == kPack) ? load16_unaligned<kSegNT>(lp + k * kRowBytes)
                                       : load16_stream<kBufNT>(lp + k * kRowBytes);
            });
        } else {
            static_for<kDepth>([&](auto k) {
                const int r = ((k - pad) % kDepth + kDepth) % kDepth;
                q[k] = u32x4{0, 0, 0, 0};
                if (r < R) q[k] = load_row(r);
            });
        }
    }

    // How many whole groups fit into n_rows rows / into the rest of a segment.
    auto groups_in = [&](uint64_t bytes) { return static_cast<int>(bytes / (uint64_t(kNE) * kRowBytes)); };

    int g = 0;
    while (g < groups) {
        const int r0 = g * kNE - pad;  // first row of the group (negative: virtual rows)
        // Steady run: n consecutive groups whose rows are real, whose kNE prefetched rows exist
        // and come from one segment (pack), and whose rows go to one segment (restore).
        int n = 0;
        const uint8_t* lp = chunks + row_offset(r0 + kDepth) + lane16;  // rows to prefetch
        const uint8_t* sp = chunks + row_offset(r0) + lane16;           // rows to write
        if (r0 >= 0 && r0 + kDepth + kNE <= R) {
            n = (R - kDepth - r0) / kNE;
            if (MODE == kPack) {
                const uint64_t s = row_offset(r0 + kDepth);
                if (span_in_segment(cin, s, kNE, &lp)) {
                    const int m = groups_in(cin.b - s);
                    n = n < m ? n : m;
                } else {
                    n = 0;
                }
            }
            if (MODE == kRestore && n > 0) {
                const uint64_t s = row_offset(r0);
                if (span_in_segment(cout, s, kNE, &sp)) {
                    const int m = groups_in(cout.b - s);
                    n = n < m ? n : m;
                } else {
                    n = 0;
                }
            }
        }
        if (n > 0) {
            uint8_t* wp = const_cast<uint8_t*>(sp);
            for (int i = 0; i < n; i++) {
                static_for<kNE>([&](auto Jc) {
                    constexpr int J = Jc;
                    const u32x4 w = q[J % kDepth];
                    if (MODE == kPack) store16_stream<kBufNT>(wp + J * kRowBytes, w);
                    if (MODE == kRestore) store16_unaligned<kSegNT>(wp + J * kRowBytes, w);
                    fold_word<J>(S, w);
                    // the refill is issued after the last use of w and the rows stay in program
                    // order, so the slot is reloaded in place and kDepth loads stay in flight
                    __builtin_amdgcn_sched_barrier(0);
                    q[J % kDepth] = (MODE == kPack) ? load16_unaligned<kSegNT>(lp + J * kRowBytes)
                                                    : load16_stream<kBufNT>(lp + J * kRowBytes);
                    __builtin_amdgcn_sched_barrier(0);
                });
                lp += kNE * kRowBytes;
                wp += kNE * kRowBytes;
            }
            g += n;
            continue;
        }
        // guarded group: virtual rows, segment boundaries, end of payload, end of tile
        static_for<kNE>([&](auto Jc) {
            constexpr int J = Jc;
            const int r = r0 + J;
            if (r >= 0) {
                const u32x4 w = q[J % kDepth];
                if (r + kDepth < R) q[J % kDepth] = load_row(r + kDepth);
                sink_row(r, w);
                fold_word<J>(S, w);
            }
        });
        g++;
    }

    if (folding) store_register(reduce_state<Fold>(S, tab, tab_u_global[1024 + lane]));
}

// Which tile a wavefront takes: position `slot` of the launch is tile tile_begin + slot of the
// buffer, or, with a chunk list, tile (slot mod tiles per chunk) of the listed chunk
// slot div tiles per chunk.  The list travels in the kernel arguments, so a call needs no device
// memory of its own for it.
template <int MODE, int HINT>
__global__ __launch_bounds__(kWaveSize* kWavesPerBlock) __attribute__((amdgpu_waves_per_eu(2))) void
tile_kernel(
    const uint64_t* __restrict__ seg_off, const uint64_t* __restrict__ seg_ptr,
    const uint32_t* __restrict__ tile_first_seg, const uint32_t* __restrict__ tab_u_global,
    uint32_t* __restrict__ partial, uint32_t* __restrict__ acc, uint8_t* __restrict__ chunks,
    TileTables T)
{
    __shared__ uint32_t tab[1024];
    __shared__ __align__(16) uint32_t ring[MODE == kRestore ? kWavesPerBlock : 1][kRingWords];
    for (int i = threadIdx.x; i < 1024; i += blockDim.x) tab[i] = tab_u_global[i];
    __syncthreads();
    const int lane = threadIdx.x & (kWaveSize - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    const uint32_t slot = xcd_order(blockIdx.x, gridDim.x, T.xcd_group) * kWavesPerBlock + wave;
    if (slot >= (T.n_list ? T.n_list : T.n_tiles)) return;
    const uint32_t tile = T.tile_begin + slot;
    if (T.skip_bad && __builtin_amdgcn_readfirstlane(T.skip_bad[tile >> T.tpc_log2])) return;
    tile_body<MODE, HINT>(seg_off, seg_ptr, tile_first_seg, tab_u_global, partial, acc, chunks, T, tab,
                          MODE == kRestore ? ring[wave] : nullptr, tile, lane);
}

template <int MODE>
__global__ __launch_bounds__(kWaveSize* kWavesPerBlock) void tile_kernel_listed(
    const uint64_t* __restrict__ seg_off, const uint64_t* __restrict__ seg_ptr,
    const uint32_t* __restrict__ tile_first_seg, const uint32_t* __restrict__ tab_u_global,
    uint32_t* __restrict__ acc, uint8_t* __restrict__ chunks, TileTables T, ChunkList list)
{
    __shared__ uint32_t tab[1024];
    for (int i = threadIdx.x; i < 1024; i += blockDim.x) tab[i] = tab_u_global[i];
    __syncthreads();
    const int lane = threadIdx.x & (kWaveSize - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    const uint32_t slot = blockIdx.x * kWavesPerBlock + wave;
    if (slot >= (list.n << T.tpc_log2)) return;
    const uint32_t chunk = list.id[slot >> T.tpc_log2];
    const uint32_t tile = (chunk << T.tpc_log2) + (slot & (T.tiles_per_chunk - 1));
    if (T.skip_bad && __builtin_amdgcn_readfirstlane(T.skip_bad[chunk])) return;
    tile_body<MODE, 3>(seg_off, seg_ptr, tile_first_seg, tab_u_global, nullptr, acc, chunks, T, tab,
                       nullptr, tile, lane);
}

// ---- per-chunk kernels around the tiles ---------------------------------------------------------

__device__ __forceinline__ uint32_t chunk_register(const uint32_t* __restrict__ partial,
                                                   uint64_t first, uint32_t n, uint32_t x_tile)
{
    uint32_t acc = 0;
    for (uint32_t i = 0; i < n; i++) acc = gf2_mul(acc, x_tile) ^ partial[first + i];
    return gf2_mul_const<kX32>(acc);  // the tiles' registers are stored without their factor x^32
}

// Before the tiles: word j of the caller's output array is set to what the tiles' registers of
// chunk j are XORed into.  Pack: the preset/complement term of a chunk-long CRC, so that the sum
// is the chunk's CRC32C.  Verify: that term XOR the stored CRC, so that the sum is zero exactly
// when the recomputed CRC equals the stored one; *n_bad is cleared as well.  The listed forms
// touch only the chunks named in the list they get as a kernel argument.
__global__ void preset_kernel(uint32_t* __restrict__ out, const uint32_t* __restrict__ crcs,
                              uint64_t first, uint64_t n, uint32_t affine,
                              uint64_t* __restrict__ n_bad)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i == 0 && n_bad) *n_bad = 0;
    if (i >= n) return;
    out[first + i] = crcs ? (affine ^ crcs[first + i]) : affine;
}

__global__ void preset_listed_kernel(uint32_t* __restrict__ out, const uint32_t* __restrict__ crcs,
                                     uint32_t affine, uint64_t* __restrict__ n_bad, ChunkList list)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0 && n_bad) *n_bad = 0;
    if (i >= list.n) return;
    const uint32_t j = list.id[i];
    out[j] = crcs ? (affine ^ crcs[j]) : affine;
}

// After the tiles of a verify pass: bad[j] becomes 0 or 1 and *n_bad counts the ones (one atomic
// per wavefront that found any).
__device__ __forceinline__ void finish_one(uint32_t* __restrict__ bad, bool valid, uint64_t j,
                                           uint64_t* __restrict__ n_bad)
{
    bool is_bad = false;
    if (valid) {
        is_bad = bad[j] != 0;
        bad[j] = is_bad ? 1u : 0u;
    }
    const unsigned long long votes = __ballot(is_bad);
    if (votes && (threadIdx.x & (kWaveSize - 1)) == 0)
        atomicAdd(reinterpret_cast<unsigned long long*>(n_bad),
                  static_cast<unsigned long long>(__popcll(votes)));
}

__global__ void finish_verify_kernel(uint32_t* __restrict__ bad, uint64_t n,
                                     uint64_t* __restrict__ n_bad)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    finish_one(bad, i < n, i, n_bad);
}

__global__ void finish_verify_listed_kernel(uint32_t* __restrict__ bad,
                                            uint64_t* __restrict__ n_bad, ChunkList list)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    finish_one(bad, i < list.n, i < list.n ? list.id[i] : 0u, n_bad);
}

__global__ void finish_crc_kernel(const uint32_t* __restrict__ partial, uint32_t n_tiles,
                                  uint32_t x_tile, const uint8_t* __restrict__ tail,
                                  uint32_t tail_bytes, uint32_t affine, uint32_t* __restrict__ out)
{
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    uint32_t c = chunk_register(partial, 0, n_tiles, x_tile);
    for (uint32_t i = 0; i < tail_bytes; i++) {
        c ^= tail[i];
        for (int k = 0; k < 8; k++) c = gf2_mulx(c);
    }
    *out = c ^ affine;
}

__global__ void zero_u64_kernel(uint64_t* p) { *p = 0; }

// Verify pass over a whole buffer, one workgroup per chunk: wavefront w folds the w-th of WAVES
// equal shares of the chunk as one message (blocks of kVerifyRows rows, straight-line), the
// shares' registers meet in LDS, and one lane compares the chunk's CRC32C with the stored one and
// writes bad[j].  No atomics on the per-chunk words and no kernels before or after it (a tile's
// register delivered by an atomic keeps its wavefront waiting for the acknowledgement, which a pass
// without stores to wait for anyway pays in full); *n_bad must be zero at launch and is touched
// for bad chunks only.  share_shift[w] = x^(32 + 8 * bytes behind share w in the chunk).
template <int WAVES, bool NT>
__global__ __launch_bounds__(kWaveSize * WAVES) void verify_chunk_kernel(
    const uint8_t* __restrict__ chunks, const uint32_t* __restrict__ tab_u_global,
    const uint32_t* __restrict__ tile_shift, uint32_t tiles_per_share, uint32_t blocks_per_share,
    uint64_t chunk_bytes, uint32_t affine, const uint32_t* __restrict__ crcs,
    uint32_t* __restrict__ bad, uint64_t* __restrict__ n_bad)
{
    __shared__ uint32_t tab[1024];
    __shared__ uint32_t regs[WAVES];
    for (int i = threadIdx.x; i < 1024; i += blockDim.x) tab[i] = tab_u_global[i];
    __syncthreads();
    const int lane = threadIdx.x & (kWaveSize - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    const uint64_t j = blockIdx.x;
    const uint32_t shift = tile_shift[(wave + 1) * tiles_per_share - 1];
    const uint8_t* bp = chunks + j * chunk_bytes +
                        static_cast<uint64_t>(wave) * blocks_per_share * (kVerifyRows * kRowBytes) +
                        16u * lane;
    uint32_t S[kNE][kNF];
    static_for<kNE>([&](auto e) { static_for<kNF>([&](auto f) { S[e][f] = 0; }); });
    constexpr int kD = kWholeDepth<kVerify>;
    for (uint32_t blk = 0; blk < blocks_per_share; blk++) {
        u32x4 w[kD];
        static_for<kD>([&](auto k) { w[k] = load16_stream<NT>(bp + k * kRowBytes); });
        static_for<kVerifyRows>([&](auto Jc) {
            constexpr int J = Jc;
            const u32x4 x = w[J % kD];
            fold_word<J % kNE>(S, x);
            if constexpr (J + kD < kVerifyRows) {
                __builtin_amdgcn_sched_barrier(0);
                w[J % kD] = load16_stream<NT>(bp + (J + kD) * kRowBytes);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        bp += kVerifyRows * kRowBytes;
    }
    const uint32_t reg = gf2_mul(reduce_state<Fold>(S, tab, tab_u_global[1024 + lane]), shift);
    if (lane == 0) regs[wave] = reg;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t crc = affine;
#pragma unroll
        for (int w = 0; w < WAVES; w++) crc ^= regs[w];
        const bool is_bad = crc != crcs[j];
        bad[j] = is_bad ? 1u : 0u;
        if (is_bad) atomicAdd(reinterpret_cast<unsigned long long*>(n_bad), 1ull);
    }
}

// Plain copy in the tile kernel's access pattern, without the CRC: 32 KiB per wavefront with 16
// rows in flight, 4 wavefronts per workgroup on adjacent tiles, XCD-aware order.  The reference
// that pack and restore are measured against.  n16 counts 16-byte units.
constexpr int kCopyRows = 32, kCopyDepth = 16;
__global__ __launch_bounds__(kWaveSize * kWavesPerBlock) void copy_kernel(
    u32x4* __restrict__ dst, const u32x4* __restrict__ src, uint64_t n16)
{
    const uint32_t lane = threadIdx.x & (kWaveSize - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    const uint64_t tile = uint64_t(xcd_order(blockIdx.x, gridDim.x, kDefaultXcdGroup)) * kWavesPerBlock + wave;
    const uint64_t i0 = tile * (kCopyRows * kWaveSize);
    if (i0 >= n16) return;
    if (i0 + kCopyRows * kWaveSize <= n16) {
        const u32x4* const s = src + i0 + lane;
        u32x4* const d = dst + i0 + lane;
        u32x4 w[kCopyDepth];
        static_for<kCopyDepth>([&](auto k) { w[k] = __builtin_nontemporal_load(s + k * kWaveSize); });
        static_for<kCopyRows>([&](auto Jc) {
            constexpr int J = Jc;
            __builtin_nontemporal_store(w[J % kCopyDepth], d + J * kWaveSize);
            if constexpr (J + kCopyDepth < kCopyRows) {
                __builtin_amdgcn_sched_barrier(0);
                w[J % kCopyDepth] = __builtin_nontemporal_load(s + (J + kCopyDepth) * kWaveSize);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    } else {
        for (uint64_t i = i0 + lane; i < n16; i += kWaveSize)
            __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
    }
}

}  // namespace

// ---- host wrappers -----------------------------------------------------------------------------

void build_tab_u(uint32_t* tab)
{
    const uint32_t u = gf2_xpow(8192);
    for (int k = 0; k < 4; k++)
        for (uint32_t b = 0; b < 256; b++) tab[k * 256 + b] = gf2_mul(b << (8 * k), u);
    for (int lane = 0; lane < 64; lane++) tab[1024 + lane] = gf2_xpow(128ull * (63 - lane));
}

template <int MODE>
static void launch_tiles_hint(int hint, dim3 grid, dim3 block, hipStream_t stream, const TileTables& t,
                              uint8_t* c)
{
#define FF_LAUNCH(H)                                                                             \
    hipLaunchKernelGGL((tile_kernel<MODE, H>), grid, block, 0, stream, t.seg_off, t.seg_ptr,      \
                       t.tile_first_seg, t.tab_u, t.partial, t.acc, c, t)
    switch (hint & 3) {
    case 0: FF_LAUNCH(0); break;
    case 1: FF_LAUNCH(1); break;
    case 2: FF_LAUNCH(2); break;
    default: FF_LAUNCH(3); break;
    }
#undef FF_LAUNCH
}

hipError_t launch_tiles(TileMode mode, const TileTables& t, void* chunks, hipStream_t stream,
                        const ChunkList* list)
{
    const dim3 block(kWaveSize * kWavesPerBlock);
    uint8_t* c = static_cast<uint8_t*>(chunks);
    if (list) {
        // listed chunks (restore and verify only): tiles of the plan's own size, default hints
        const uint64_t count = static_cast<uint64_t>(list->n) << t.tpc_log2;
        if (count == 0) return hipSuccess;
        if (mode == kPack || t.partial || list->n > kMaxListedChunks || count > 0x7FFFFFF0ull)
            return hipErrorInvalidValue;
        const dim3 grid(static_cast<unsigned>((count + kWavesPerBlock - 1) / kWavesPerBlock));
        if (mode == kRestore)
            hipLaunchKernelGGL((tile_kernel_listed<kRestore>), grid, block, 0, stream, t.seg_off,
                               t.seg_ptr, t.tile_first_seg, t.tab_u, t.acc, c, t, *list);
        else
            hipLaunchKernelGGL((tile_kernel_listed<kVerify>), grid, block, 0, stream, t.seg_off,
                               t.seg_ptr, t.tile_first_seg, t.tab_u, t.acc, c, t, *list);
        return hipGetLastError();
    }
    const uint32_t count = t.n_list ? t.n_list : t.n_tiles;
    if (count == 0) return hipSuccess;
    const dim3 grid((count + kWavesPerBlock - 1) / kWavesPerBlock);
    switch (mode) {
    case kPack: launch_tiles_hint<kPack>(t.hint, grid, block, stream, t, c); break;
    case kRestore: launch_tiles_hint<kRestore>(t.hint, grid, block, stream, t, c); break;
    case kVerify: launch_tiles_hint<kVerify>(t.hint, grid, block, stream, t, c); break;
    }
    return hipGetLastError();
}

hipError_t launch_preset(uint32_t* out, const uint32_t* crcs, uint64_t first, uint64_t n,
                         uint32_t affine, uint64_t* n_bad, const ChunkList* list,
                         hipStream_t stream)
{
    const uint64_t count = list ? list->n : n;
    const unsigned block = 256;
    unsigned grid = static_cast<unsigned>((count + block - 1) / block);
    if (grid == 0) grid = 1;  // *n_bad is cleared even when there is no chunk to preset
    if (list)
        hipLaunchKernelGGL(preset_listed_kernel, dim3(grid), dim3(block), 0, stream, out, crcs,
                           affine, n_bad, *list);
    else
        hipLaunchKernelGGL(preset_kernel, dim3(grid), dim3(block), 0, stream, out, crcs, first, n,
                           affine, n_bad);
    return hipGetLastError();
}

hipError_t launch_finish_verify(uint32_t* bad, uint64_t n, uint64_t* n_bad, const ChunkList* list,
                                hipStream_t stream)
{
    const uint64_t count = list ? list->n : n;
    if (count == 0) return hipSuccess;
    const unsigned block = 256;
    const unsigned grid = static_cast<unsigned>((count + block - 1) / block);
    if (list)
        hipLaunchKernelGGL(finish_verify_listed_kernel, dim3(grid), dim3(block), 0, stream, bad,
                           n_bad, *list);
    else
        hipLaunchKernelGGL(finish_verify_kernel, dim3(grid), dim3(block), 0, stream, bad, n, n_bad);
    return hipGetLastError();
}

hipError_t launch_finish_crc(const uint32_t* partial, uint32_t n_tiles, uint32_t x_tile,
                             const uint8_t* tail, uint32_t tail_bytes, uint32_t affine,
                             uint32_t* out, hipStream_t stream)
{
    hipLaunchKernelGGL(finish_crc_kernel, dim3(1), dim3(64), 0, stream, partial, n_tiles, x_tile,
                       tail, tail_bytes, affine, out);
    return hipGetLastError();
}

bool verify_chunks_applicable(uint64_t chunk_bytes, uint64_t n_chunks)
{
    // every wavefront needs whole 64 KiB blocks, and the launch enough wavefronts to fill the chip
    return chunk_bytes >= 4ull * kVerifyRows * kRowBytes && n_chunks * 4 >= 4096 &&
           n_chunks <= 0x7FFFFFFFull;
}

hipError_t launch_verify_chunks(const TileTables& t, uint64_t chunk_bytes, uint32_t tile_bytes,
                                uint32_t plan_tiles_per_chunk, uint32_t affine, const void* chunks,
                                const uint32_t* crcs, uint32_t* bad, uint64_t* n_bad,
                                uint64_t n_chunks, hipStream_t stream)
{
    if (!verify_chunks_applicable(chunk_bytes, n_chunks)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, stream, n_bad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const uint8_t* c = static_cast<const uint8_t*>(chunks);
    const bool nt = (t.hint & 2) != 0;
    // 8 wavefronts per chunk once a share of an eighth is still 1 MiB, else 4
    const uint32_t waves = chunk_bytes >= (8ull << 20) ? 8 : 4;
    const uint64_t share = chunk_bytes / waves;
    const uint32_t tiles_per_share = plan_tiles_per_chunk / waves;  // plan tiles are <= 32 KiB here
    const uint32_t blocks_per_share = static_cast<uint32_t>(share / (kVerifyRows * kRowBytes));
    if (tiles_per_share == 0 || uint64_t(tiles_per_share) * tile_bytes != share)
        return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(n_chunks));
#define FF_VLAUNCH(W, NT)                                                                         \
    hipLaunchKernelGGL((verify_chunk_kernel<W, NT>), grid, dim3(kWaveSize* W), 0, stream, c, t.tab_u, \
                       t.tile_shift, tiles_per_share, blocks_per_share, chunk_bytes, affine, crcs,   \
                       bad, n_bad)
    if (waves == 8) {
        if (nt) FF_VLAUNCH(8, true); else FF_VLAUNCH(8, false);
    } else {
        if (nt) FF_VLAUNCH(4, true); else FF_VLAUNCH(4, false);
    }
#undef FF_VLAUNCH
    return hipGetLastError();
}

hipError_t launch_zero_u64(uint64_t* p, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, uint64_t nbytes, hipStream_t stream)
{
    const uint64_t n16 = nbytes / 16;
    if (n16 == 0) return hipSuccess;
    const uint64_t tiles = (n16 + kCopyRows * kWaveSize - 1) / (kCopyRows * kWaveSize);
    const uint64_t blocks = (tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
    hipLaunchKernelGGL(copy_kernel, dim3(static_cast<unsigned>(blocks)),
                       dim3(kWaveSize * kWavesPerBlock), 0, stream, static_cast<u32x4*>(dst),
                       static_cast<const u32x4*>(src), n16);
    return hipGetLastError();
}

}  // namespace ffsnap
