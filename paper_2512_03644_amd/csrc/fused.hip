// Fused optimizer step + snapshot for gfx950.
//
// Work tiles (layout.hpp) are runs of up to kParamTileElems elements of one parameter group, one
// workgroup each, and runs of up to kRawTileBytes of a RAW segment, one wavefront each in a
// kernel of their own that only copies and folds.  A parameter tile is walked in rows of 256
// elements, lane l taking 4 consecutive elements: 8 bytes of 16-bit gradient and 3 x 16 bytes of
// fp32 master/m/v come in, the AdamW update runs in registers, and the four results go out
// twice -- in place, and at their stream offsets in the chunk buffer -- plus once into LDS,
// from where four folding wavefronts (one per output stream) take them into their CRC states,
// so the snapshot is never read back from memory.  Rows are aligned to the END of the tile: a
// tile whose length is not a multiple of 256 has a partial FIRST row, whose missing leading
// elements are zeros that do not change a CRC register started from 0.  At the end of the tile
// each stream's state is reduced to a register, multiplied by x^(8 * distance to the end of its
// chunk) and XORed into crcs[chunk] with an atomic; XOR is commutative, so the result does not
// depend on the order in which tiles finish.  A prepare kernel sets crcs[] to the preset/complement
// term and writes the zero tail of the last chunk.
#include "fused.hpp"

#include <hip/hip_fp16.h>

#include "fold.h"

namespace ffsnap {

namespace {

constexpr int kUpdateWaves = 4;  // one row of a batch each
constexpr int kFoldWaves = 4;    // one output stream each
constexpr int kWavesPerBlock = kUpdateWaves + kFoldWaves;
constexpr int kBatchRows = kUpdateWaves;
using F32Fold = Fold16x16;  // 16 bytes per lane per row (parameter tiles)
using B16Fold = Fold8x20;   // 8 bytes per lane per row
using RawFold = Fold16x10;  // RAW copy tiles
constexpr int kPhases = 5;  // rows folded between two physical rotations of the state
static_assert(kPhases <= RawFold::NE, "rotation step");
constexpr int kRowElems = 256;
constexpr int kRawRows = kRawTileBytes / 1024;  // rows of a whole RAW tile
constexpr int kRawDepth = 16;                   // rows in flight on its straight-line path
static_assert(kRawRows % F32Fold::NE == 0 && kRawDepth <= kRawRows, "whole RAW tile");

__device__ __forceinline__ float bits_to_f32(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f32_to_bits(float f) { return __float_as_uint(f); }

// fp32 -> bf16 bits, round to nearest even; NaN keeps sign and top payload bits, forced quiet.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t u = f32_to_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// fp32 -> fp16 bits: the hardware conversion rounds to nearest even, overflows to infinity and
// produces subnormals; NaN is given a fixed form (sign, top 9 payload bits, quiet).
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f)
{
    const uint32_t u = f32_to_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return ((u >> 16) & 0x8000u) | 0x7E00u | ((u >> 13) & 0x1FFu);
    return __half_as_ushort(__float2half_rn(f));
}

// IEEE 754 leaves sign and payload of a NaN that an operation produces open, and processors differ
// in them.  A snapshot is compared byte for byte and CRC'd across machines, so a NaN result of the
// update is stored in one form: quiet, positive, empty payload.
constexpr uint32_t kCanonicalNaN = 0x7FC00000u;
__device__ __forceinline__ float canonical_nan(float x) { return (x != x) ? bits_to_f32(kCanonicalNaN) : x; }

// One element of the update; every operation is a separately rounded fp32 operation (the file
// is compiled with -ffp-contract=off, division and square root are correctly rounded).  New
// master, m and v that are NaN are stored as the canonical NaN, and the 16-bit weight is rounded
// from that.
// F16: the gradient is fp16 of a loss scaled by S and is multiplied by inv_scale = 1/S first;
// the working weight is rounded to fp16.  Otherwise both are bf16 and nothing is scaled.
template <bool F16>
__device__ __forceinline__ void adam_element(const FusedConsts& C, uint32_t g_bits, float& p,
                                             float& m, float& v, uint32_t& w_bits)
{
    const AdamConsts& k = C.adam;
    float g;
    if constexpr (F16)
        g = __half2float(__ushort_as_half(static_cast<unsigned short>(g_bits))) * C.inv_scale;
    else
        g = bits_to_f32(g_bits << 16);
    const float pd = p * k.decay;
    const float m1 = (k.b1 * m) + (k.omb1 * g);
    const float v1 = (k.b2 * v) + ((k.omb2 * g) * g);
    // x / 1.0f is x exactly, so the division is skipped once the second bias correction has
    // rounded to one (wave-uniform test; beta2 = 0.95 gets there at step 333)
    const float r = sqrtf(v1);
    const float d = ((k.bc2s == 1.0f) ? r : (r / k.bc2s)) + k.eps;
    const float p1 = canonical_nan(pd - (k.step_size * (m1 / d)));
    p = p1;
    m = canonical_nan(m1);
    v = canonical_nan(v1);
    w_bits = F16 ? f32_to_f16_bits(p1) : f32_to_bf16_bits(p1);
}

// fp16 infinity or NaN
__device__ __forceinline__ bool f16_nonfinite(uint32_t bits) { return (bits & 0x7C00u) == 0x7C00u; }

struct Lds {
    uint32_t tab16[1024];  // multiply by x^8192  (1 KiB rows)
    uint32_t tab8[1024];   // multiply by x^4096  (512 B rows)
    uint32_t lane16[64];   // x^(128 * (63 - lane))
    uint32_t lane8[64];    // x^(64 * (63 - lane))
};

// Tile registers come out of reduce_state without the factor x^32 that a CRC register carries.
constexpr uint32_t kX16 = gf2_xpow(16);

__device__ __forceinline__ void add_piece(uint32_t* __restrict__ crcs, const WorkTile& t, int piece,
                                          uint32_t reg)
{
    if (t.shift[piece])
        atomicXor(&crcs[t.chunk[piece]], gf2_mul_const<kX32>(gf2_mul(reg, t.shift[piece])));
}

// Head piece: the first two bytes of a split element, which are the last two bytes of their
// chunk.  In the low half of a dword they read M(x) * x^16, and their register is M(x) * x^32.
__device__ __forceinline__ void add_head_piece(uint32_t* __restrict__ crcs, const WorkTile& t,
                                               int piece, uint32_t low_half)
{
    atomicXor(&crcs[t.chunk[piece]], gf2_mul_const<kX16>(low_half));
}

// ---- parameter tile ----------------------------------------------------------------------------
//
// A workgroup of 8 wavefronts owns one parameter tile.  Wavefronts 0..3 update: in every batch of
// 4 rows each takes one row, runs the AdamW update in registers, stores the results twice (in
// place, snapshot) and leaves a copy in LDS.  Wavefronts 4..7 fold: each owns ONE output stream
// (w16, master, m, v) and one CRC state, and folds the 4 rows of the previous batch out of LDS.
// One barrier per batch separates writers and readers of the two LDS batch buffers.  Splitting
// the roles keeps every wavefront's register set small (one fold state instead of four), which
// lets several wavefronts share a SIMD and overlap arithmetic with memory waits.

struct Batch {          // results of 4 rows, as they lie in the streams
    uint32_t w[kBatchRows][128];
    uint32_t p[kBatchRows][256];
    uint32_t m[kBatchRows][256];
    uint32_t v[kBatchRows][256];
};

struct RowIn {
    u32x2 g;
    u32x4 p, m, v;
};

struct TileGeom {
    int n, pad_el, rows, n_batches, pad_rows;
};

__device__ __forceinline__ TileGeom tile_geom(const WorkTile& t)
{
    TileGeom g;
    g.n = static_cast<int>(t.n);
    g.pad_el = (kRowElems - g.n % kRowElems) % kRowElems;  // elements missing in front of row 0
    g.rows = (g.n + g.pad_el) / kRowElems;
    g.n_batches = (g.rows + kBatchRows - 1) / kBatchRows;
    g.pad_rows = g.n_batches * kBatchRows - g.rows;  // virtual zero rows in front of row 0
    return g;
}

// Update wavefront `u` (0..3): rows u - pad_rows, u - pad_rows + 4, ...
//
// Only the first of these rows can be virtual or partial; it is handled before the loop.  From
// then on every row is full, so the loop has no branch around a memory access: its loads are
// unconditional and refill, in place, the register set whose values were just taken out (two sets,
// for even and odd batches).  Registers that are never copied while a load into them is in flight,
// and no branch between issue and use, let the compiler wait for exactly the loads a row needs,
// while the loads of the next batch and the stores of the last one stay in flight.
template <bool F16, bool CHAINED>
__device__ __forceinline__ void update_role(const WorkTile& t, const TileGeom& G,
                                            const uint8_t* __restrict__ grad,
                                            uint8_t* __restrict__ chunks,
                                            uint32_t* __restrict__ crcs, const FusedConsts& C,
                                            Batch (&buf)[2], int u, int lane)
{
    uint8_t* const tw = reinterpret_cast<uint8_t*>(t.ptr[0]);
    uint8_t* const tp = reinterpret_cast<uint8_t*>(t.ptr[1]);
    uint8_t* const tm = reinterpret_cast<uint8_t*>(t.ptr[2]);
    uint8_t* const tv = reinterpret_cast<uint8_t*>(t.ptr[3]);
    const uint8_t* const tg = grad + 2 * t.e0;
    uint8_t* const sw = chunks + t.soff[0];
    uint8_t* const sp = chunks + t.soff[1];
    uint8_t* const sm = chunks + t.soff[2];
    uint8_t* const sv = chunks + t.soff[3];
    // where the old master, m, v come from: their tensors, or the previous snapshot
    const uint8_t* const lp = CHAINED ? C.prev + t.soff[1] : tp;
    const uint8_t* const lm = CHAINED ? C.prev + t.soff[2] : tm;
    const uint8_t* const lv = CHAINED ? C.prev + t.soff[3] : tv;
    uint32_t nonfinite = 0;  // this lane's count of infinite or NaN gradient elements (fp16 only)

    // A row can use vector accesses if every lane holds 4 real elements.
    auto full_row = [&](int r) { return r > 0 || (r == 0 && G.pad_el == 0); };
    auto load_row = [&](int r, RowIn& in) {  // r must be a full row of the tile
        const int j0 = r * kRowElems + 4 * lane - G.pad_el;
        in.g = load8_unaligned<true>(tg + 2 * j0);
        in.p = load16_unaligned<true>(lp + 4 * j0);
        in.m = load16_unaligned<true>(lm + 4 * j0);
        in.v = load16_unaligned<true>(lv + 4 * j0);
    };

    // copy of a row's results for the folding wavefronts, which fold them and store the full rows
    auto publish = [&](Batch& out, uint32_t (&fw)[2], uint32_t (&fp)[4], uint32_t (&fm)[4],
                       uint32_t (&fv)[4]) {
        *reinterpret_cast<u32x2*>(&out.w[u][2 * lane]) = u32x2{fw[0], fw[1]};
        *reinterpret_cast<u32x4*>(&out.p[u][4 * lane]) = u32x4{fp[0], fp[1], fp[2], fp[3]};
        *reinterpret_cast<u32x4*>(&out.m[u][4 * lane]) = u32x4{fm[0], fm[1], fm[2], fm[3]};
        *reinterpret_cast<u32x4*>(&out.v[u][4 * lane]) = u32x4{fv[0], fv[1], fv[2], fv[3]};
    };

    // a full row from registers
    auto full_row_step = [&](Batch& out, const RowIn& cur) {
        uint32_t gb[4], wb[4];
        float p[4], m[4], v[4];
        gb[0] = cur.g.x & 0xFFFFu; gb[1] = cur.g.x >> 16;
        gb[2] = cur.g.y & 0xFFFFu; gb[3] = cur.g.y >> 16;
        p[0] = bits_to_f32(cur.p.x); p[1] = bits_to_f32(cur.p.y);
        p[2] = bits_to_f32(cur.p.z); p[3] = bits_to_f32(cur.p.w);
        m[0] = bits_to_f32(cur.m.x); m[1] = bits_to_f32(cur.m.y);
        m[2] = bits_to_f32(cur.m.z); m[3] = bits_to_f32(cur.m.w);
        v[0] = bits_to_f32(cur.v.x); v[1] = bits_to_f32(cur.v.y);
        v[2] = bits_to_f32(cur.v.z); v[3] = bits_to_f32(cur.v.w);
#pragma unroll
        for (int s = 0; s < 4; s++) {
            if constexpr (F16) nonfinite += f16_nonfinite(gb[s]) ? 1u : 0u;
            adam_element<F16>(C, gb[s], p[s], m[s], v[s], wb[s]);
        }
        uint32_t fw[2] = {wb[0] | (wb[1] << 16), wb[2] | (wb[3] << 16)};
        uint32_t fp[4], fm[4], fv[4];
#pragma unroll
        for (int s = 0; s < 4; s++) {
            fp[s] = f32_to_bits(p[s]);
            fm[s] = f32_to_bits(m[s]);
            fv[s] = f32_to_bits(v[s]);
        }
        publish(out, fw, fp, fm, fv);
    };

    // the partial first row of a tile: element by element; absent elements stay zero
    auto partial_row_step = [&](Batch& out, int r) {
        const int j0 = r * kRowElems + 4 * lane - G.pad_el;
        uint32_t gb[4], wb[4];
        float p[4], m[4], v[4];
#pragma unroll
        for (int s = 0; s < 4; s++) {
            const int j = j0 + s;
            gb[s] = 0; wb[s] = 0; p[s] = 0.f; m[s] = 0.f; v[s] = 0.f;
            if (j >= 0) {
                gb[s] = *as_global(reinterpret_cast<const uint16_t*>(tg + 2 * j));
                if constexpr (CHAINED) {
                    // stream offsets of fp32 segments may be 2 mod 4: halfword loads
                    auto f32_at = [](const uint8_t* q) {
                        const uint16_t* h = reinterpret_cast<const uint16_t*>(q);
                        return bits_to_f32(uint32_t(*as_global(h)) | (uint32_t(*as_global(h + 1)) << 16));
                    };
                    p[s] = f32_at(lp + 4 * j);
                    m[s] = f32_at(lm + 4 * j);
                    v[s] = f32_at(lv + 4 * j);
                } else {
                    p[s] = *as_global(reinterpret_cast<const float*>(tp + 4 * j));
                    m[s] = *as_global(reinterpret_cast<const float*>(tm + 4 * j));
                    v[s] = *as_global(reinterpret_cast<const float*>(tv + 4 * j));
                }
                if constexpr (F16) nonfinite += f16_nonfinite(gb[s]) ? 1u : 0u;
                adam_element<F16>(C, gb[s], p[s], m[s], v[s], wb[s]);
                *as_global(reinterpret_cast<uint16_t*>(tw + 2 * j)) = static_cast<uint16_t>(wb[s]);
                if constexpr (!CHAINED) {
                    *as_global(reinterpret_cast<float*>(tp + 4 * j)) = p[s];
                    *as_global(reinterpret_cast<float*>(tm + 4 * j)) = m[s];
                    *as_global(reinterpret_cast<float*>(tv + 4 * j)) = v[s];
                }
                *as_global(reinterpret_cast<uint16_t*>(sw + 2 * j)) = static_cast<uint16_t>(wb[s]);
                // stream offsets of fp32 segments may be 2 mod 4: halfword stores
                const uint32_t pb = f32_to_bits(p[s]), mb = f32_to_bits(m[s]), vb = f32_to_bits(v[s]);
                uint16_t* qp = reinterpret_cast<uint16_t*>(sp + 4 * j);
                uint16_t* qm = reinterpret_cast<uint16_t*>(sm + 4 * j);
                uint16_t* qv = reinterpret_cast<uint16_t*>(sv + 4 * j);
                *as_global(qp) = static_cast<uint16_t>(pb);
                *as_global(qp + 1) = static_cast<uint16_t>(pb >> 16);
                *as_global(qm) = static_cast<uint16_t>(mb);
                *as_global(qm + 1) = static_cast<uint16_t>(mb >> 16);
                *as_global(qv) = static_cast<uint16_t>(vb);
                *as_global(qv + 1) = static_cast<uint16_t>(vb >> 16);
            }
        }
        uint32_t fw[2] = {wb[0] | (wb[1] << 16), wb[2] | (wb[3] << 16)};
        uint32_t fp[4], fm[4], fv[4];
#pragma unroll
        for (int s = 0; s < 4; s++) {
            fp[s] = f32_to_bits(p[s]);
            fm[s] = f32_to_bits(m[s]);
            fv[s] = f32_to_bits(v[s]);
        }
        publish(out, fw, fp, fm, fv);
    };

    const int first = u - G.pad_rows;  // this wavefront's row of batch 0
    const int nb = G.n_batches;
    int b = 0;
    if (!full_row(first)) {
        // a virtual row (zeros) or the partial first row of the tile
        if (first < 0) {
            uint32_t zw[2] = {0, 0}, z4[4] = {0, 0, 0, 0};
            publish(buf[0], zw, z4, z4, z4);
        } else {
            partial_row_step(buf[0], first);
        }
        __syncthreads();  // the barrier of batch 0
        b = 1;
    }
    // rows first + 4b', b' >= b, are full rows
    RowIn qa, qb;  // inputs of batch b, b + 2, ... and of batch b + 1, b + 3, ...
    qa = qb = RowIn{u32x2{0, 0}, u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}};
    if (b < nb) load_row(first + kBatchRows * b, qa);
    if (b + 1 < nb) load_row(first + kBatchRows * (b + 1), qb);
    // one batch: take the inputs out of `q`, refill `q` for two batches later, update the row
    auto batch_step = [&](int bb, RowIn& q, auto prefetch_c) {
        const int r = first + kBatchRows * bb;
        const RowIn cur = q;
        if constexpr (decltype(prefetch_c)::value) load_row(r + 2 * kBatchRows, q);
        full_row_step(buf[bb & 1], cur);
        __syncthreads();
    };
    // steady part: the batches two ahead exist.  Its first round stands in front of the loop, so
    // that the loop is entered with the same loads and stores in flight as on its back edge.
    if (b + 3 < nb) {
        batch_step(b, qa, std::true_type{});
        batch_step(b + 1, qb, std::true_type{});
        b += 2;
    }
    while (b + 3 < nb) {
        batch_step(b, qa, std::true_type{});
        batch_step(b + 1, qb, std::true_type{});
        b += 2;
    }
    // up to three batches are left; only the first of three still has something to prefetch
    const int left = nb - b;
    if (left == 3) {
        batch_step(b, qa, std::true_type{});
        batch_step(b + 1, qb, std::false_type{});
        batch_step(b + 2, qa, std::false_type{});
    } else if (left == 2) {
        batch_step(b, qa, std::false_type{});
        batch_step(b + 1, qb, std::false_type{});
    } else if (left == 1) {
        batch_step(b, qa, std::false_type{});
    }
    __syncthreads();  // the folding wavefronts take the last batch after this one

    if constexpr (F16) {
        if (C.n_nonfinite) {
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) nonfinite += __shfl_xor(nonfinite, d);
            if (lane == 0 && nonfinite)
                atomicAdd(reinterpret_cast<unsigned long long*>(C.n_nonfinite),
                          static_cast<unsigned long long>(nonfinite));
        }
    }
}

// Folding wavefront of stream x (0 = w16, 1..3 = master, m, v): takes the rows of the previous
// batch out of LDS, stores every full row to the snapshot and (if `tensor` is set) in place, and
// folds it.  A wavefront thus sweeps two store streams that carry the same bytes, instead of every
// updating wavefront scattering its row over eight; the partial first row of a tile is stored
// element by element by the updating wavefront that produced it.
template <class F, int DW>
__device__ __forceinline__ uint32_t fold_stream(const WorkTile& t, const TileGeom& G,
                                                Batch (&buf)[2], int x, int lane,
                                                uint8_t* __restrict__ tensor,
                                                uint8_t* __restrict__ snap,
                                                uint32_t* __restrict__ crcs, const uint32_t* tab,
                                                const uint32_t* lane_tab)
{
    constexpr int NE = F::NE;
    static_assert(NE % kBatchRows == 0 && F::NF == DW, "a batch never straddles the rotation");
    uint32_t S[NE][DW];
    static_for<NE>([&](auto e) { static_for<DW>([&](auto f) { S[e][f] = 0; }); });
    const int head_lane = G.pad_el / 4, head_sub = G.pad_el % 4;  // where element 0 sits in row 0
    auto store_row = [&](int r, const uint32_t (&d)[DW]) {
        const int j0 = r * kRowElems + 4 * lane - G.pad_el;  // first element of the lane
        if constexpr (DW == 2) {
            const u32x2 w = {d[0], d[1]};
            if (tensor) store8_unaligned<true>(tensor + 2 * j0, w);
            store8_unaligned<true>(snap + 2 * j0, w);
        } else {
            const u32x4 w = {d[0], d[1], d[2], d[3]};
            if (tensor) store16_unaligned<true>(tensor + 4 * j0, w);
            store16_unaligned<true>(snap + 4 * j0, w);
        }
    };
    // start the rotation so that it is back at zero after the last batch
    int phase = (NE - (G.n_batches * kBatchRows) % NE) % NE;
    for (int b = 0; b <= G.n_batches; b++) {
        if (b >= 1) {
            const Batch& in = buf[(b - 1) & 1];
            uint32_t d[kBatchRows][DW];
            static_for<kBatchRows>([&](auto k) {
                const uint32_t* row = (DW == 2) ? &in.w[k][2 * lane]
                                                : (x == 1 ? &in.p[k][4 * lane]
                                                          : (x == 2 ? &in.m[k][4 * lane] : &in.v[k][4 * lane]));
                static_for<DW>([&](auto f) { d[k][f] = row[f]; });
            });
            const int r0 = (b - 1) * kBatchRows - G.pad_rows;  // tile row of the batch's first row
            if (b == 1) {
                // the first batch may hold virtual rows (r < 0) and the partial row (r == 0)
                static_for<kBatchRows>([&](auto k) {
                    const int r = r0 + k;
                    if (r > 0 || (r == 0 && G.pad_el == 0)) store_row(r, d[k]);
                    // split first element: its first two bytes close the previous chunk and
                    // must not enter this tile's CRC of that stream
                    if (DW == 4 && r == 0 && (t.head_split & (1u << x)) && lane == head_lane) {
                        static_for<DW>([&](auto sc) {
                            if (sc == head_sub) {
                                // two message bytes in the low half are M(x) * x^16; their
                                // register is M(x) * x^32
                                add_head_piece(crcs, t, 3 + x, d[k][sc] & 0xFFFFu);
                                d[k][sc] &= 0xFFFF0000u;
                            }
                        });
                    }
                });
            } else {
                static_for<kBatchRows>([&](auto k) { store_row(r0 + k, d[k]); });
            }
            static_for<NE / kBatchRows>([&](auto Qc) {
                constexpr int Q = Qc;
                if (phase == Q * kBatchRows) {
                    static_for<kBatchRows>([&](auto k) { fold_row<F, Q * kBatchRows + k>(S, d[k]); });
                }
            });
            phase = (phase + kBatchRows) % NE;
        }
        __syncthreads();
    }
    return reduce_state<F>(S, tab, lane_tab[lane]);  // tables are complete after any barrier
}

// ---- RAW tile: plain copy into the snapshot -----------------------------------------------------

__device__ __forceinline__ void run_raw_tile(const WorkTile& t, uint8_t* __restrict__ chunks,
                                             uint32_t* __restrict__ crcs, const Lds& lds, int lane)
{
    const int n = static_cast<int>(t.n);  // bytes, even
    const uint8_t* const src = reinterpret_cast<const uint8_t*>(t.ptr[0]);
    uint8_t* const dst = chunks + t.soff[0];
    if (n == kRawRows * 1024) {
        // a whole tile: straight-line code, kRawDepth rows in flight
        uint32_t S[F32Fold::NE][4];
        static_for<F32Fold::NE>([&](auto e) { static_for<4>([&](auto f) { S[e][f] = 0; }); });
        u32x4 w[kRawDepth];
        static_for<kRawDepth>(
            [&](auto k) { w[k] = load16_unaligned<true>(src + k * 1024 + 16 * lane); });
        static_for<kRawRows>([&](auto Jc) {
            constexpr int J = Jc;
            const u32x4 x = w[J % kRawDepth];
            store16_unaligned<true>(dst + J * 1024 + 16 * lane, x);
            const uint32_t d[4] = {x.x, x.y, x.z, x.w};
            fold_row<F32Fold, J % F32Fold::NE>(S, d);
            if constexpr (J + kRawDepth < kRawRows) {
                __builtin_amdgcn_sched_barrier(0);
                w[J % kRawDepth] = load16_unaligned<true>(src + (J + kRawDepth) * 1024 + 16 * lane);
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        const uint32_t reg = reduce_state<F32Fold>(S, lds.tab16, lds.lane16[lane]);
        if (lane == 0) add_piece(crcs, t, 0, reg);
        return;
    }
    constexpr int NE = RawFold::NE;
    const int pad_b = (1024 - n % 1024) % 1024;
    const int rows = (n + pad_b) / 1024;
    const int pad_rows = (kPhases - rows % kPhases) % kPhases;

    uint32_t S[NE][4];
    static_for<NE>([&](auto e) { static_for<4>([&](auto f) { S[e][f] = 0; }); });
    for (int r = 0; r < rows; r++) {
        const int b0 = r * 1024 + 16 * lane - pad_b;
        uint32_t d[4] = {0, 0, 0, 0};
        if (b0 >= 0) {
            const u32x4 w = load16_unaligned<true>(src + b0);
            store16_unaligned<true>(dst + b0, w);
            d[0] = w.x; d[1] = w.y; d[2] = w.z; d[3] = w.w;
        } else {
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const int b = b0 + 2 * u;
                if (b >= 0) {
                    const uint32_t h = *as_global(reinterpret_cast<const uint16_t*>(src + b));
                    *as_global(reinterpret_cast<uint16_t*>(dst + b)) = static_cast<uint16_t>(h);
                    d[u >> 1] |= h << ((u & 1) * 16);
                }
            }
        }
        const int phase = (r + pad_rows) % kPhases;
        static_for<kPhases>([&](auto Jc) {
            constexpr int J = Jc;
            if (phase == J) {
                fold_row<RawFold, J>(S, d);
                if constexpr (J == kPhases - 1) rotate_state<RawFold, kPhases>(S);
            }
        });
    }
    const uint32_t reg = reduce_state<RawFold>(S, lds.tab16, lds.lane16[lane]);
    if (lane == 0) add_piece(crcs, t, 0, reg);
}

// The gradient pointers of the parameter groups [grad_base, grad_base + kGradsPerLaunch) travel by
// value in the kernel arguments: the step keeps no per-call table in device memory, so calls on
// one plan may overlap and a captured launch carries its own pointers.
template <bool F16, bool CHAINED>
__global__ __launch_bounds__(kWaveSize* kWavesPerBlock) void fused_kernel(
    const WorkTile* __restrict__ tiles, uint32_t n_tiles, uint32_t grad_base,
    const uint32_t* __restrict__ tabs, uint8_t* __restrict__ chunks, uint32_t* __restrict__ crcs,
    FusedConsts C, GradPtrs grads)
{
    __shared__ Lds lds;
    __shared__ Batch buf[2];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    const uint32_t ti = xcd_order(blockIdx.x, gridDim.x, C.xcd_group);  // one tile per workgroup
    if (ti >= n_tiles) return;
    // The reduction tables are used after the last barrier of a tile only (every tile passes at
    // least two), so the folding wavefronts fetch them while the updating wavefronts are already
    // loading their first rows.
    if (wave >= kUpdateWaves) {
        for (int i = threadIdx.x - kUpdateWaves * kWaveSize; i < 1024; i += kFoldWaves * kWaveSize) {
            lds.tab16[i] = tabs[i];
            lds.tab8[i] = tabs[1024 + i];
        }
        if (wave == kUpdateWaves) {
            lds.lane16[lane] = tabs[2048 + lane];
            lds.lane8[lane] = tabs[2048 + 64 + lane];
        }
    }
    // the tile descriptor is uniform and read-only: the loads below go through scalar registers
    // (a private copy indexed by the stream number would live in scratch memory instead)
    const WorkTile& t = tiles[ti];
    if (t.kind != kWorkParam) return;  // RAW tiles belong to raw_kernel
    // every wavefront of the workgroup passes the same n_batches + 1 barriers
    const TileGeom G = tile_geom(t);
    if (wave < kUpdateWaves) {
        const uint8_t* grad = reinterpret_cast<const uint8_t*>(grads.p[t.grad_index - grad_base]);
        update_role<F16, CHAINED>(t, G, grad, chunks, crcs, C, buf, wave, lane);
    } else {
        const int x = wave - kUpdateWaves;
        uint8_t* const snap = chunks + t.soff[x];
        uint32_t reg;
        if (x == 0) {
            reg = fold_stream<B16Fold, 2>(t, G, buf, x, lane, reinterpret_cast<uint8_t*>(t.ptr[0]),
                                          snap, crcs, lds.tab8, lds.lane8);
        } else {
            // chained step: master, m and v live in the snapshots only
            uint8_t* const tensor = CHAINED ? nullptr : reinterpret_cast<uint8_t*>(t.ptr[x]);
            reg = fold_stream<F32Fold, 4>(t, G, buf, x, lane, tensor, snap, crcs, lds.tab16,
                                          lds.lane16);
        }
        if (lane == 0) add_piece(crcs, t, x, reg);
    }
}

// ---- the step's traffic alone (bench helper) -------------------------------------------------------
//
// The loads and stores of a parameter tile with no arithmetic and no CRC, in the shape that moved
// this mix of streams fastest in microbenchmarks: a workgroup of 4 wavefronts stages half a tile
// (at most 4096 elements, 56 KiB) in LDS in two phases.  Load: the 1 KiB rows of the four input
// streams -- gradient, master, m, v -- form one list that is cut into four equal runs, and every
// wavefront requests its run up front, so a wavefront sweeps contiguous memory of one or two
// streams.  Store: the rows of the eight output streams -- in place x 4, snapshot x 4 -- form one
// list cut the same way.  The new 16-bit weights are the gradient's bits; master, m, v keep their
// values.  Overlap of loads and stores comes from the two workgroups a CU holds being in different
// phases.  (With the update and the CRC added this shape loses to fused_kernel: a tile must fit
// LDS whole, which halves it, and the per-tile reductions and the update, done in phases of their
// own, then take more ALU time per element than the memory phases leave.)
// Every stream's image in LDS is aligned to its END: a stream of nbytes takes rows = ceil(nbytes /
// 1 KiB) rows and starts pad = rows * 1 KiB - nbytes bytes into its first row.

constexpr int kStageWaves = 4;
constexpr int kStageThreads = kStageWaves * kWaveSize;
constexpr int kStageElems = 4096;
constexpr int kRowsF = kStageElems * 4 / 1024;  // rows of a whole fp32 stream of a half tile
constexpr int kRowsW = kStageElems * 2 / 1024;  // rows of a whole 16-bit stream
constexpr int kRowsIn = kRowsW + 3 * kRowsF;
static_assert(kRowsIn % kStageWaves == 0, "whole half tiles split evenly");
static_assert(kParamTileElems <= 2 * kStageElems, "a parameter tile is staged in two halves");

struct StageGeom {
    int n;               // elements
    int rows_w, rows_f;  // rows of the 16-bit stream / of each fp32 stream
    int pad_w, pad_f;    // bytes in front of the data in row 0
};

// byte offset of stream x's image (0: w16 / gradient, 1..3: master, m, v) in LDS
__device__ __forceinline__ int stage_base(int x)
{
    return x == 0 ? 0 : kRowsW * 1024 + (x - 1) * kRowsF * 1024;
}

template <bool CHAINED>
__global__ __launch_bounds__(kStageThreads) void mix_ceiling_kernel(
    const WorkTile* __restrict__ tiles, uint32_t n_tiles, uint32_t grad_base,
    uint8_t* __restrict__ chunks, FusedConsts C, GradPtrs grads)
{
    __shared__ __attribute__((aligned(16))) uint8_t img[kRowsIn * 1024];
    const int lane = threadIdx.x & (kWaveSize - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    // workgroup position p: half p mod 2 of tile p div 2
    const uint32_t pos = xcd_order(blockIdx.x, gridDim.x, C.xcd_group);
    const uint32_t ti = pos / 2;
    if (ti >= n_tiles) return;
    const WorkTile& t = tiles[ti];
    if (t.kind != kWorkParam) return;
    const int e_off = static_cast<int>(pos % 2) * kStageElems;  // first element of this half
    if (e_off >= static_cast<int>(t.n)) return;
    StageGeom G;
    G.n = static_cast<int>(t.n) - e_off < kStageElems ? static_cast<int>(t.n) - e_off : kStageElems;
    G.rows_w = (2 * G.n + 1023) / 1024;
    G.rows_f = (4 * G.n + 1023) / 1024;
    G.pad_w = G.rows_w * 1024 - 2 * G.n;
    G.pad_f = G.rows_f * 1024 - 4 * G.n;
    const uint32_t lane16 = 16u * lane;
    auto elem_bytes = [](int x) { return x == 0 ? 2 : 4; };

    // ---- load ------------------------------------------------------------------------------------
    {
        // where stream x is read from: the gradient; master, m, v from their tensors or, chained,
        // from the previous snapshot at their stream offsets
        const uint8_t* src[4];
        src[0] = reinterpret_cast<const uint8_t*>(grads.p[t.grad_index - grad_base]) +
                 2 * (t.e0 + e_off);
#pragma unroll
        for (int x = 1; x < 4; x++)
            src[x] = (CHAINED ? C.prev + t.soff[x] : reinterpret_cast<const uint8_t*>(t.ptr[x])) +
                     4 * e_off;
        const int total = G.rows_w + 3 * G.rows_f;
        const int per = (total + kStageWaves - 1) / kStageWaves;
        constexpr int kPer = kRowsIn / kStageWaves;
        u32x4 q[kPer];
        // row i of this wavefront's run: which stream, which row of it (x < 0: none)
        auto decode = [&](int i, int& x, int& r) {
            const int rr = wave * per + i;
            x = -1;
            r = rr;
            if (i < per && rr < total) {
                x = 0;
                if (r >= G.rows_w) {
                    r -= G.rows_w;
                    x = 1;
                    if (r >= G.rows_f) { r -= G.rows_f; x = 2; }
                    if (r >= G.rows_f) { r -= G.rows_f; x = 3; }
                }
            }
        };
        static_for<kPer>([&](auto ic) {
            constexpr int i = ic;
            int x, r;
            decode(i, x, r);
            q[i] = u32x4{0, 0, 0, 0};
            if (x >= 0) {
                const uint8_t* sp = x == 0 ? src[0] : (x == 1 ? src[1] : (x == 2 ? src[2] : src[3]));
                const int pad = x == 0 ? G.pad_w : G.pad_f;
                const int off = r * 1024 + static_cast<int>(lane16) - pad;  // in the stream's data
                if (off >= 0) {
                    q[i] = load16_unaligned<true>(sp + off);
                } else if (off > -16) {
                    // the lane's 16 bytes begin in the pad (row 0 only): halfword by halfword
                    uint32_t h[8];
#pragma unroll
                    for (int u = 0; u < 8; u++) {
                        const int b = off + 2 * u;
                        h[u] = b >= 0 ? *as_global(reinterpret_cast<const uint16_t*>(sp + b)) : 0u;
                    }
                    q[i] = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16),
                                 h[6] | (h[7] << 16)};
                }
            }
        });
        static_for<kPer>([&](auto ic) {
            constexpr int i = ic;
            int x, r;
            decode(i, x, r);
            if (x >= 0) *reinterpret_cast<u32x4*>(&img[stage_base(x) + r * 1024 + lane16]) = q[i];
        });
    }
    __syncthreads();

    // ---- store -----------------------------------------------------------------------------------
    {
        // The output streams in the order their rows are listed: in place master, m, v (not when
        // chained), in place w16, then snapshot master, m, v, w16.  o counts through that list;
        // stream_of(o) is the image it is taken from.
        constexpr int kOut = CHAINED ? 5 : 8;
        constexpr int kInPlace = CHAINED ? 1 : 4;
        auto stream_of = [&](int o) {
            return o < kInPlace ? (o == kInPlace - 1 ? 0 : o + 1) : ((o - kInPlace + 1) & 3);
        };
        auto rows_of = [&](int o) { return stream_of(o) == 0 ? G.rows_w : G.rows_f; };
        const int total = (kOut - 2) * G.rows_f + 2 * G.rows_w;
        const int per = (total + kStageWaves - 1) / kStageWaves;
        constexpr int kPer = 2 * kRowsIn / kStageWaves;
        // this wavefront's run starts at row r of output stream o
        int o = 0, r = wave * per;
        static_for<kOut>([&](auto) {
            if (o < kOut && r >= rows_of(o)) {
                r -= rows_of(o);
                o++;
            }
        });
        static_for<kPer>([&](auto ic) {
            constexpr int i = ic;
            if (i < per && o < kOut) {
                const int x = stream_of(o);
                const int pad = x == 0 ? G.pad_w : G.pad_f;
                uint8_t* const d = (o < kInPlace ? reinterpret_cast<uint8_t*>(t.ptr[x]) : chunks + t.soff[x]) +
                                   elem_bytes(x) * e_off;
                const u32x4 w = *reinterpret_cast<const u32x4*>(&img[stage_base(x) + r * 1024 + lane16]);
                const int off = r * 1024 + static_cast<int>(lane16) - pad;
                if (off >= 0) {
                    store16_unaligned<true>(d + off, w);
                } else if (off > -16) {
                    const uint32_t dd[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                    for (int u = 0; u < 8; u++) {
                        const int b = off + 2 * u;
                        if (b >= 0)
                            *as_global(reinterpret_cast<uint16_t*>(d + b)) =
                                static_cast<uint16_t>(dd[u >> 1] >> ((u & 1) * 16));
                    }
                }
                r++;
                if (r >= rows_of(o)) {
                    r = 0;
                    o++;
                }
            }
        });
    }
}

// RAW tiles: one wavefront per tile copies its bytes into the snapshot and folds them.
constexpr int kRawWaves = 4;
__global__ __launch_bounds__(kWaveSize* kRawWaves) void raw_kernel(
    const WorkTile* __restrict__ tiles, uint32_t n_tiles, const uint32_t* __restrict__ tabs,
    uint8_t* __restrict__ chunks, uint32_t* __restrict__ crcs)
{
    __shared__ Lds lds;
    for (int i = threadIdx.x; i < 1024; i += blockDim.x) lds.tab16[i] = tabs[i];
    if (threadIdx.x < kWaveSize) lds.lane16[threadIdx.x] = tabs[2048 + threadIdx.x];
    __syncthreads();
    const int lane = threadIdx.x & (kWaveSize - 1);
    // consecutive tiles per XCD, as in the tile kernel (a RAW tile is a 32 KiB copy as well)
    const uint32_t ti = xcd_order(blockIdx.x, gridDim.x, kDefaultXcdGroup) * kRawWaves +
                        __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    if (ti >= n_tiles) return;
    const WorkTile& t = tiles[ti];
    if (t.kind != kWorkRaw) return;
    run_raw_tile(t, chunks, crcs, lds, lane);
}

// crcs[] = the preset/complement term (the tiles XOR their pieces into it), the tail of the last
// chunk = 0, and the non-finite gradient counter = 0
__global__ void fused_prepare_kernel(uint32_t* __restrict__ crcs, uint64_t n_chunks, uint32_t affine,
                                     uint8_t* __restrict__ chunks, uint64_t payload,
                                     uint64_t buffer_bytes, uint64_t* __restrict__ n_nonfinite)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i == 0 && n_nonfinite) *n_nonfinite = 0;
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
    for (uint64_t j = i; j < n_chunks; j += stride) crcs[j] = affine;
    uint16_t* tail = reinterpret_cast<uint16_t*>(chunks + payload);  // payload is even
    const uint64_t n_half = (buffer_bytes - payload) / 2;
    for (uint64_t j = i; j < n_half; j += stride) tail[j] = 0;
}

}  // namespace

void build_fused_tabs(uint32_t* tab)
{
    const uint64_t row_bytes[2] = {1024, 512};
    for (int t = 0; t < 2; t++) {
        const uint32_t u = gf2_xpow(8 * row_bytes[t]);
        for (int k = 0; k < 4; k++)
            for (uint32_t b = 0; b < 256; b++) tab[t * 1024 + k * 256 + b] = gf2_mul(b << (8 * k), u);
        for (int lane = 0; lane < 64; lane++)
            tab[2048 + t * 64 + lane] = gf2_xpow(8 * (row_bytes[t] / 64) * (63 - lane));
    }
}

hipError_t launch_fused(bool f16, const WorkTile* tiles, uint32_t n_param_tiles,
                        uint32_t n_raw_tiles, const void* const* grads, uint32_t n_params,
                        const uint32_t* group_tile_begin, const uint32_t* tabs, void* chunks,
                        uint32_t* crcs, uint64_t n_chunks, uint64_t payload, uint64_t buffer_bytes,
                        uint32_t affine, const FusedConsts& consts, bool bare, hipStream_t stream)
{
    uint8_t* c = static_cast<uint8_t*>(chunks);
    hipError_t e = hipSuccess;
    if (!bare) {
        const uint64_t prep_items = n_chunks > (buffer_bytes - payload) / 2
                                        ? n_chunks
                                        : (buffer_bytes - payload) / 2;
        unsigned prep_blocks = static_cast<unsigned>((prep_items + 255) / 256);
        if (prep_blocks == 0) prep_blocks = 1;
        if (prep_blocks > 4096) prep_blocks = 4096;
        hipLaunchKernelGGL(fused_prepare_kernel, dim3(prep_blocks), dim3(256), 0, stream, crcs,
                           n_chunks, affine, c, payload, buffer_bytes,
                           f16 ? consts.n_nonfinite : nullptr);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const bool chained = consts.prev != nullptr;
    auto kernel = chained ? (f16 ? fused_kernel<true, true> : fused_kernel<false, true>)
                          : (f16 ? fused_kernel<true, false> : fused_kernel<false, false>);
    // one launch per kGradsPerLaunch parameter groups; the parameter tiles are sorted by group
    for (uint32_t k = 0, p0 = 0; p0 < n_params && n_param_tiles; k++, p0 += kGradsPerLaunch) {
        const uint32_t t0 = group_tile_begin[k], t1 = group_tile_begin[k + 1];
        if (t1 == t0) continue;
        GradPtrs g;
        for (uint32_t i = 0; i < kGradsPerLaunch; i++)
            g.p[i] = p0 + i < n_params ? reinterpret_cast<uint64_t>(grads[p0 + i]) : 0;
        if (bare) {
            // two workgroups per tile, one per half
            if (chained)
                hipLaunchKernelGGL(mix_ceiling_kernel<true>, dim3(2 * (t1 - t0)), dim3(kStageThreads),
                                   0, stream, tiles + t0, t1 - t0, p0, c, consts, g);
            else
                hipLaunchKernelGGL(mix_ceiling_kernel<false>, dim3(2 * (t1 - t0)),
                                   dim3(kStageThreads), 0, stream, tiles + t0, t1 - t0, p0, c, consts,
                                   g);
        } else {
            hipLaunchKernelGGL(kernel, dim3(t1 - t0), dim3(kWaveSize * kWavesPerBlock), 0, stream,
                               tiles + t0, t1 - t0, p0, tabs, c, crcs, consts, g);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (n_raw_tiles && !bare) {
        const unsigned grid = (n_raw_tiles + kRawWaves - 1) / kRawWaves;
        hipLaunchKernelGGL(raw_kernel, dim3(grid), dim3(kWaveSize * kRawWaves), 0, stream,
                           tiles + n_param_tiles, n_raw_tiles, tabs, c, crcs);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace ffsnap
