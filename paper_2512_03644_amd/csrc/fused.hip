// Fused optimizer step + snapshot for gfx950.
//
// One wavefront owns one work tile (layout.hpp): a run of up to 65536 elements of one parameter
// group, or a run of bytes of a RAW segment.  A parameter tile is walked in rows of 256
// elements, lane l taking 4 consecutive elements: 8 bytes of bf16 gradient and 3 x 16 bytes of
// fp32 master/m/v come in, the AdamW update runs in registers, and the four results go out
// twice -- in place, and at their stream offsets in the chunk buffer.  The same registers feed
// four CRC folding states (three 16-byte-per-lane streams, one 8-byte-per-lane stream), so the
// snapshot is never read back.  Rows are aligned to the END of the tile: a tile whose length is
// not a multiple of 256 has a partial FIRST row, whose missing leading elements are zeros that
// do not change a CRC register started from 0.  At the end of the tile each stream's state is
// reduced to a register, multiplied by x^(8 * distance to the end of its chunk) and XORed into
// crcs[chunk] with an atomic; XOR is commutative, so the result does not depend on the order in
// which tiles finish.  A prepare kernel zeroes crcs[] and the zero tail of the last chunk; a
// finish kernel adds the preset/complement term.
#include "fused.hpp"

#include "fold.h"

namespace ffsnap {

namespace {

constexpr int kWavesPerBlock = 4;
using F32Fold = Fold16x10;  // 16 bytes per lane per row
using B16Fold = Fold8x20;   // 8 bytes per lane per row
constexpr int kPhases = 5;  // rows folded between two physical rotations of the state
static_assert(kPhases <= F32Fold::NE && kPhases <= B16Fold::NE, "rotation step");
constexpr int kRowElems = 256;
constexpr int kBatch = 1;  // rows loaded, updated and stored together

__device__ __forceinline__ float bits_to_f32(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f32_to_bits(float f) { return __float_as_uint(f); }

// fp32 -> bf16 bits, round to nearest even; NaN keeps sign and top payload bits, forced quiet.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t u = f32_to_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// One element of the update; every operation is a separately rounded fp32 operation (the file
// is compiled with -ffp-contract=off, division and square root are correctly rounded).
__device__ __forceinline__ void adam_element(const AdamConsts& k, uint32_t g_bits, float& p,
                                             float& m, float& v, uint32_t& w_bits)
{
    const float g = bits_to_f32(g_bits << 16);
    const float pd = p * k.decay;
    const float m1 = (k.b1 * m) + (k.omb1 * g);
    const float v1 = (k.b2 * v) + ((k.omb2 * g) * g);
    // x / 1.0f is x exactly, so the division is skipped once the second bias correction has
    // rounded to one (wave-uniform test; beta2 = 0.95 gets there at step 333)
    const float r = sqrtf(v1);
    const float d = ((k.bc2s == 1.0f) ? r : (r / k.bc2s)) + k.eps;
    const float p1 = pd - (k.step_size * (m1 / d));
    p = p1;
    m = m1;
    v = v1;
    w_bits = f32_to_bf16_bits(p1);
}

struct Lds {
    uint32_t tab16[1024];  // multiply by x^8192  (1 KiB rows)
    uint32_t tab8[1024];   // multiply by x^4096  (512 B rows)
};

__device__ __forceinline__ void add_piece(uint32_t* __restrict__ crcs, const WorkTile& t, int piece,
                                          uint32_t reg)
{
    if (t.shift[piece])
        atomicXor(&crcs[t.chunk[piece]], gf2_mul(reg, t.shift[piece]));
}

// ---- parameter tile ----------------------------------------------------------------------------

__device__ __forceinline__ void run_param_tile(const WorkTile& t, const uint8_t* __restrict__ grad,
                                               uint8_t* __restrict__ chunks,
                                               uint32_t* __restrict__ crcs, const FusedConsts& C,
                                               const Lds& lds, int lane)
{
    const int n = static_cast<int>(t.n);
    const int pad_el = (kRowElems - n % kRowElems) % kRowElems;  // missing in front of row 0
    const int rows = (n + pad_el) / kRowElems;
    const int pad_rows = (kPhases - rows % kPhases) % kPhases;

    uint8_t* const tw = reinterpret_cast<uint8_t*>(t.ptr[0]);
    uint8_t* const tp = reinterpret_cast<uint8_t*>(t.ptr[1]);
    uint8_t* const tm = reinterpret_cast<uint8_t*>(t.ptr[2]);
    uint8_t* const tv = reinterpret_cast<uint8_t*>(t.ptr[3]);
    const uint8_t* const tg = grad + 2 * t.e0;
    uint8_t* const sw = chunks + t.soff[0];
    uint8_t* const sp = chunks + t.soff[1];
    uint8_t* const sm = chunks + t.soff[2];
    uint8_t* const sv = chunks + t.soff[3];

    uint32_t Sp[F32Fold::NE][4], Sm[F32Fold::NE][4], Sv[F32Fold::NE][4], Sw[B16Fold::NE][2];
    static_for<F32Fold::NE>([&](auto e) {
        static_for<4>([&](auto f) { Sp[e][f] = 0; Sm[e][f] = 0; Sv[e][f] = 0; });
    });
    static_for<B16Fold::NE>([&](auto e) { Sw[e][0] = 0; Sw[e][1] = 0; });

    // lane and sub-position of element 0 (for the head pieces of split elements)
    const int head_lane = pad_el / 4, head_sub = pad_el % 4;

    struct RowIn {
        u32x2 g;
        u32x4 p, m, v;
    };
    // Only the folding step depends on how far the state registers have rotated, so it alone is
    // selected by a switch on the phase.  Unrolling a whole rotation (20 rows) would put ~90 KB
    // of code in the loop; instead the rotation is undone with register moves every kPhases
    // rows, which keeps the loop body small enough for the instruction cache.  Starting at phase
    // pad_rows makes the last row end a block, so the state ends in logical order.
    auto fold_all = [&](int r, uint32_t (&fw)[2], uint32_t (&fp)[4], uint32_t (&fm)[4],
                        uint32_t (&fv)[4]) {
        const int phase = (r + pad_rows) % kPhases;
        static_for<kPhases>([&](auto Jc) {
            constexpr int J = Jc;
            if (phase == J) {
                fold_row<B16Fold, J>(Sw, fw);
                fold_row<F32Fold, J>(Sp, fp);
                fold_row<F32Fold, J>(Sm, fm);
                fold_row<F32Fold, J>(Sv, fv);
                if constexpr (J == kPhases - 1) {
                    rotate_state<B16Fold, kPhases>(Sw);
                    rotate_state<F32Fold, kPhases>(Sp);
                    rotate_state<F32Fold, kPhases>(Sm);
                    rotate_state<F32Fold, kPhases>(Sv);
                }
            }
        });
    };
    // Update one row in registers and fold it; the row's results replace its inputs (g becomes
    // the packed bf16 weights).
    auto update_row = [&](int r, RowIn& io) {
        uint32_t gb[4] = {io.g.x & 0xFFFFu, io.g.x >> 16, io.g.y & 0xFFFFu, io.g.y >> 16};
        uint32_t wb[4];
        float p[4] = {bits_to_f32(io.p.x), bits_to_f32(io.p.y), bits_to_f32(io.p.z), bits_to_f32(io.p.w)};
        float m[4] = {bits_to_f32(io.m.x), bits_to_f32(io.m.y), bits_to_f32(io.m.z), bits_to_f32(io.m.w)};
        float v[4] = {bits_to_f32(io.v.x), bits_to_f32(io.v.y), bits_to_f32(io.v.z), bits_to_f32(io.v.w)};
#pragma unroll
        for (int s = 0; s < 4; s++) adam_element(C.adam, gb[s], p[s], m[s], v[s], wb[s]);
        uint32_t fw[2] = {wb[0] | (wb[1] << 16), wb[2] | (wb[3] << 16)};
        uint32_t fp[4] = {f32_to_bits(p[0]), f32_to_bits(p[1]), f32_to_bits(p[2]), f32_to_bits(p[3])};
        uint32_t fm[4] = {f32_to_bits(m[0]), f32_to_bits(m[1]), f32_to_bits(m[2]), f32_to_bits(m[3])};
        uint32_t fv[4] = {f32_to_bits(v[0]), f32_to_bits(v[1]), f32_to_bits(v[2]), f32_to_bits(v[3])};
        io.g = u32x2{fw[0], fw[1]};
        io.p = u32x4{fp[0], fp[1], fp[2], fp[3]};
        io.m = u32x4{fm[0], fm[1], fm[2], fm[3]};
        io.v = u32x4{fv[0], fv[1], fv[2], fv[3]};
        // split first element (row 0 of a tile that starts on a full row): its first two bytes
        // close the previous chunk
        if (r == 0 && t.head_split && lane == head_lane) {
            uint32_t* const fx[3] = {fp, fm, fv};
#pragma unroll
            for (int x = 1; x <= 3; x++) {
                if (t.head_split & (1u << x)) {
                    const uint32_t d = fx[x - 1][0];  // pad_el == 0 here: element 0 is sub 0
                    // two message bytes in the low half are M(x) * x^16; their register is
                    // M(x) * x^32
                    add_piece(crcs, t, 3 + x, gf2_mul(d & 0xFFFFu, C.x16));
                    fx[x - 1][0] = d & 0xFFFF0000u;
                }
            }
        }
        fold_all(r, fw, fp, fm, fv);
    };

    int r_first = 0;
    if (pad_el != 0) {
        // partial first row: element by element; absent elements stay zero and fold as zeros
        r_first = 1;
        const int j0 = 4 * lane - pad_el;
        uint32_t gb[4], wb[4];
        float p[4], m[4], v[4];
#pragma unroll
        for (int s = 0; s < 4; s++) {
            const int j = j0 + s;
            gb[s] = 0; wb[s] = 0; p[s] = 0.f; m[s] = 0.f; v[s] = 0.f;
            if (j >= 0) {
                gb[s] = *as_global(reinterpret_cast<const uint16_t*>(tg + 2 * j));
                p[s] = *as_global(reinterpret_cast<const float*>(tp + 4 * j));
                m[s] = *as_global(reinterpret_cast<const float*>(tm + 4 * j));
                v[s] = *as_global(reinterpret_cast<const float*>(tv + 4 * j));
                adam_element(C.adam, gb[s], p[s], m[s], v[s], wb[s]);
                *as_global(reinterpret_cast<uint16_t*>(tw + 2 * j)) = static_cast<uint16_t>(wb[s]);
                *as_global(reinterpret_cast<float*>(tp + 4 * j)) = p[s];
                *as_global(reinterpret_cast<float*>(tm + 4 * j)) = m[s];
                *as_global(reinterpret_cast<float*>(tv + 4 * j)) = v[s];
                *as_global(reinterpret_cast<uint16_t*>(sw + 2 * j)) = static_cast<uint16_t>(wb[s]);
                // stream offsets of fp32 segments may be 2 mod 4: halfword stores
                const uint32_t pb = f32_to_bits(p[s]), mb = f32_to_bits(m[s]), vb = f32_to_bits(v[s]);
                uint16_t* qp = reinterpret_cast<uint16_t*>(sp + 4 * j);
                uint16_t* qm = reinterpret_cast<uint16_t*>(sm + 4 * j);
                uint16_t* qv = reinterpret_cast<uint16_t*>(sv + 4 * j);
                qp[0] = static_cast<uint16_t>(pb); qp[1] = static_cast<uint16_t>(pb >> 16);
                qm[0] = static_cast<uint16_t>(mb); qm[1] = static_cast<uint16_t>(mb >> 16);
                qv[0] = static_cast<uint16_t>(vb); qv[1] = static_cast<uint16_t>(vb >> 16);
            }
        }
        uint32_t fw[2] = {wb[0] | (wb[1] << 16), wb[2] | (wb[3] << 16)};
        uint32_t fp[4] = {f32_to_bits(p[0]), f32_to_bits(p[1]), f32_to_bits(p[2]), f32_to_bits(p[3])};
        uint32_t fm[4] = {f32_to_bits(m[0]), f32_to_bits(m[1]), f32_to_bits(m[2]), f32_to_bits(m[3])};
        uint32_t fv[4] = {f32_to_bits(v[0]), f32_to_bits(v[1]), f32_to_bits(v[2]), f32_to_bits(v[3])};
        if (t.head_split && lane == head_lane) {
            uint32_t* const fx[3] = {fp, fm, fv};
#pragma unroll
            for (int x = 1; x <= 3; x++) {
                if (t.head_split & (1u << x)) {
#pragma unroll
                    for (int s = 0; s < 4; s++) {
                        if (s == head_sub) {
                            const uint32_t d = fx[x - 1][s];
                            add_piece(crcs, t, 3 + x, gf2_mul(d & 0xFFFFu, C.x16));
                            fx[x - 1][s] = d & 0xFFFF0000u;
                        }
                    }
                }
            }
        }
        fold_all(0, fw, fp, fm, fv);
    }

    // Full rows in batches of kBatch.  Per batch and per stream the kBatch loads, and later the
    // kBatch stores, are issued back to back, so each stream presents 4 KiB of consecutive
    // addresses to the memory system at a time (measured: +10 % bandwidth over row-by-row
    // issue).  The inputs of the next batch are requested before the current one is updated.
    // Loads past the last row are redirected to the last row (always in bounds, never used).
    if (r_first < rows) {
        auto load_batch = [&](RowIn (&q)[kBatch], int r0) {
            static_for<kBatch>([&](auto k) {
                const int rr = r0 + k;
                const int j0 = (rr < rows ? rr : rows - 1) * kRowElems + 4 * lane - pad_el;
                q[k].g = load8_unaligned<true>(tg + 2 * j0);
            });
            static_for<kBatch>([&](auto k) {
                const int rr = r0 + k;
                const int j0 = (rr < rows ? rr : rows - 1) * kRowElems + 4 * lane - pad_el;
                q[k].p = load16_unaligned<true>(tp + 4 * j0);
            });
            static_for<kBatch>([&](auto k) {
                const int rr = r0 + k;
                const int j0 = (rr < rows ? rr : rows - 1) * kRowElems + 4 * lane - pad_el;
                q[k].m = load16_unaligned<true>(tm + 4 * j0);
            });
            static_for<kBatch>([&](auto k) {
                const int rr = r0 + k;
                const int j0 = (rr < rows ? rr : rows - 1) * kRowElems + 4 * lane - pad_el;
                q[k].v = load16_unaligned<true>(tv + 4 * j0);
            });
        };
        RowIn cur[kBatch], nxt[kBatch];
        load_batch(nxt, r_first);
        for (int r0 = r_first; r0 < rows; r0 += kBatch) {
            static_for<kBatch>([&](auto k) { cur[k] = nxt[k]; });
            load_batch(nxt, r0 + kBatch);
            // one copy of the update code: rows rotate through cur[0], results queue up behind
            for (int k = 0; k < kBatch; k++) {
                RowIn x = cur[0];
                static_for<kBatch - 1>([&](auto i) { cur[i] = cur[i + 1]; });
                if (r0 + k < rows) update_row(r0 + k, x);
                cur[kBatch - 1] = x;
            }
            const int nb = rows - r0;  // real rows in this batch (>= kBatch except at the end)
            auto j0_of = [&](int k) { return (r0 + k) * kRowElems + 4 * lane - pad_el; };
            static_for<kBatch>([&](auto k) { if (k < nb) store8_unaligned(tw + 2 * j0_of(k), cur[k].g); });
            static_for<kBatch>([&](auto k) { if (k < nb) store16_unaligned(tp + 4 * j0_of(k), cur[k].p); });
            static_for<kBatch>([&](auto k) { if (k < nb) store16_unaligned(tm + 4 * j0_of(k), cur[k].m); });
            static_for<kBatch>([&](auto k) { if (k < nb) store16_unaligned(tv + 4 * j0_of(k), cur[k].v); });
            static_for<kBatch>([&](auto k) { if (k < nb) store8_unaligned<true>(sw + 2 * j0_of(k), cur[k].g); });
            static_for<kBatch>([&](auto k) { if (k < nb) store16_unaligned<true>(sp + 4 * j0_of(k), cur[k].p); });
            static_for<kBatch>([&](auto k) { if (k < nb) store16_unaligned<true>(sm + 4 * j0_of(k), cur[k].m); });
            static_for<kBatch>([&](auto k) { if (k < nb) store16_unaligned<true>(sv + 4 * j0_of(k), cur[k].v); });
        }
    }

    const uint32_t rw = reduce_state<B16Fold>(Sw, lds.tab8, C.x32, C.z8);
    const uint32_t rp = reduce_state<F32Fold>(Sp, lds.tab16, C.x32, C.z16);
    const uint32_t rm = reduce_state<F32Fold>(Sm, lds.tab16, C.x32, C.z16);
    const uint32_t rv = reduce_state<F32Fold>(Sv, lds.tab16, C.x32, C.z16);
    if (lane == 0) {
        add_piece(crcs, t, 0, rw);
        add_piece(crcs, t, 1, rp);
        add_piece(crcs, t, 2, rm);
        add_piece(crcs, t, 3, rv);
    }
}

// ---- RAW tile: plain copy into the snapshot -----------------------------------------------------

__device__ __forceinline__ void run_raw_tile(const WorkTile& t, uint8_t* __restrict__ chunks,
                                             uint32_t* __restrict__ crcs, const FusedConsts& C,
                                             const Lds& lds, int lane)
{
    constexpr int NE = F32Fold::NE;
    const int n = static_cast<int>(t.n);  // bytes, even
    const int pad_b = (1024 - n % 1024) % 1024;
    const int rows = (n + pad_b) / 1024;
    const int pad_rows = (kPhases - rows % kPhases) % kPhases;
    const uint8_t* const src = reinterpret_cast<const uint8_t*>(t.ptr[0]);
    uint8_t* const dst = chunks + t.soff[0];

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
                fold_row<F32Fold, J>(S, d);
                if constexpr (J == kPhases - 1) rotate_state<F32Fold, kPhases>(S);
            }
        });
    }
    const uint32_t reg = reduce_state<F32Fold>(S, lds.tab16, C.x32, C.z16);
    if (lane == 0) add_piece(crcs, t, 0, reg);
}

__global__ __launch_bounds__(kWaveSize* kWavesPerBlock) void fused_kernel(
    const WorkTile* __restrict__ tiles, uint32_t n_tiles, const uint64_t* __restrict__ grads,
    const uint32_t* __restrict__ tabs, uint8_t* __restrict__ chunks, uint32_t* __restrict__ crcs,
    FusedConsts C)
{
    __shared__ Lds lds;
    for (int i = threadIdx.x; i < 1024; i += blockDim.x) {
        lds.tab16[i] = tabs[i];
        lds.tab8[i] = tabs[1024 + i];
    }
    __syncthreads();
    const int lane = threadIdx.x & (kWaveSize - 1);
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWaveSize);
    const uint32_t ti = blockIdx.x * kWavesPerBlock + wave;
    if (ti >= n_tiles) return;
    // the tile descriptor is wave-uniform: read it through scalar registers
    WorkTile t;
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(tiles + ti);
        uint32_t* dst = reinterpret_cast<uint32_t*>(&t);
#pragma unroll
        for (unsigned i = 0; i < sizeof(WorkTile) / 4; i++)
            dst[i] = __builtin_amdgcn_readfirstlane(src[i]);
    }
    if (t.kind == kWorkParam) {
        const uint8_t* grad = reinterpret_cast<const uint8_t*>(grads[t.grad_index]);
        run_param_tile(t, grad, chunks, crcs, C, lds, lane);
    } else {
        run_raw_tile(t, chunks, crcs, C, lds, lane);
    }
}

// crcs[] = 0 and the tail of the last chunk = 0
__global__ void fused_prepare_kernel(uint32_t* __restrict__ crcs, uint64_t n_chunks,
                                     uint8_t* __restrict__ chunks, uint64_t payload,
                                     uint64_t buffer_bytes)
{
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    const uint64_t stride = static_cast<uint64_t>(gridDim.x) * blockDim.x;
    for (uint64_t j = i; j < n_chunks; j += stride) crcs[j] = 0;
    uint16_t* tail = reinterpret_cast<uint16_t*>(chunks + payload);  // payload is even
    const uint64_t n_half = (buffer_bytes - payload) / 2;
    for (uint64_t j = i; j < n_half; j += stride) tail[j] = 0;
}

__global__ void fused_finish_kernel(uint32_t* __restrict__ crcs, uint64_t n_chunks, uint32_t affine)
{
    const uint64_t j = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (j < n_chunks) crcs[j] ^= affine;
}

}  // namespace

void build_tab(uint32_t* tab, uint64_t row_bytes)
{
    const uint32_t u = gf2_xpow(8 * row_bytes);
    for (int k = 0; k < 4; k++)
        for (uint32_t b = 0; b < 256; b++) tab[k * 256 + b] = gf2_mul(b << (8 * k), u);
}

void fill_fused_crc_consts(FusedConsts& c)
{
    c.x32 = gf2_xpow(32);
    c.x16 = gf2_xpow(16);
    for (int l = 0; l < 6; l++) {
        c.z16[l] = gf2_xpow(128ull << l);
        c.z8[l] = gf2_xpow(64ull << l);
    }
}

hipError_t launch_fused(const WorkTile* tiles, uint32_t n_tiles, const uint64_t* grads,
                        const uint32_t* tabs, void* chunks, uint32_t* crcs, uint64_t n_chunks,
                        uint64_t payload, uint64_t buffer_bytes, uint32_t affine,
                        const FusedConsts& consts, hipStream_t stream)
{
    uint8_t* c = static_cast<uint8_t*>(chunks);
    const uint64_t prep_items = n_chunks > (buffer_bytes - payload) / 2 ? n_chunks
                                                                         : (buffer_bytes - payload) / 2;
    unsigned prep_blocks = static_cast<unsigned>((prep_items + 255) / 256);
    if (prep_blocks == 0) prep_blocks = 1;
    if (prep_blocks > 4096) prep_blocks = 4096;
    hipLaunchKernelGGL(fused_prepare_kernel, dim3(prep_blocks), dim3(256), 0, stream, crcs, n_chunks,
                       c, payload, buffer_bytes);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (n_tiles) {
        const unsigned grid = (n_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
        hipLaunchKernelGGL(fused_kernel, dim3(grid), dim3(kWaveSize * kWavesPerBlock), 0, stream,
                           tiles, n_tiles, grads, tabs, c, crcs, consts);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(fused_finish_kernel, dim3(static_cast<unsigned>((n_chunks + 255) / 256)),
                       dim3(256), 0, stream, crcs, n_chunks, affine);
    return hipGetLastError();
}

}  // namespace ffsnap
