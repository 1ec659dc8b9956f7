// Device-side building blocks shared by the kernels: 16-byte accesses, the table-free CRC
// folding step, and the reduction of a folded state to a 32-bit CRC register.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "fold_taps.h"
#include "gf2.h"

namespace ffsnap {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef u32x2 u32x2_a2 __attribute__((aligned(2)));

// Every pointer the kernels dereference is device global memory.  Addresses that come out of
// tables are plain integers, so the compiler would fall back to flat (generic) accesses, whose
// completion order it cannot count on; casting to the global address space gives global_load /
// global_store, which complete in order and can be kept in flight with exact wait counts.
#define FF_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ FF_GLOBAL T* as_global(T* p)
{
    return (FF_GLOBAL T*)p;
}

constexpr int kWaveSize = 64;

template <class Fn, int... Is>
__device__ __forceinline__ void static_for_impl(Fn&& fn, std::integer_sequence<int, Is...>)
{
    (fn(std::integral_constant<int, Is>{}), ...);
}
template <int N, class Fn>
__device__ __forceinline__ void static_for(Fn&& fn)
{
    static_for_impl(fn, std::make_integer_sequence<int, N>{});
}

// Tensor side: 16 (or 8) bytes at any even address.  Buffer side: 16-byte aligned.  NT marks
// the access non-temporal (streaming data that will not be reused).
template <bool NT = false>
__device__ __forceinline__ u32x4 load16_unaligned(const uint8_t* p)
{
    if (NT) return __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4_a2*>(p)));
    return *as_global(reinterpret_cast<const u32x4_a2*>(p));
}
template <bool NT = false>
__device__ __forceinline__ void store16_unaligned(uint8_t* p, u32x4 w)
{
    if (NT)
        __builtin_nontemporal_store(w, as_global(reinterpret_cast<u32x4_a2*>(p)));
    else
        *as_global(reinterpret_cast<u32x4_a2*>(p)) = w;
}
template <bool NT = false>
__device__ __forceinline__ u32x2 load8_unaligned(const uint8_t* p)
{
    if (NT) return __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x2_a2*>(p)));
    return *as_global(reinterpret_cast<const u32x2_a2*>(p));
}
template <bool NT = false>
__device__ __forceinline__ void store8_unaligned(uint8_t* p, u32x2 w)
{
    if (NT)
        __builtin_nontemporal_store(w, as_global(reinterpret_cast<u32x2_a2*>(p)));
    else
        *as_global(reinterpret_cast<u32x2_a2*>(p)) = w;
}
template <bool NT = true>
__device__ __forceinline__ u32x4 load16_stream(const uint8_t* p)
{
    if (NT) return __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4*>(p)));
    return *as_global(reinterpret_cast<const u32x4*>(p));
}
template <bool NT = true>
__device__ __forceinline__ void store16_stream(uint8_t* p, u32x4 w)
{
    if (NT)
        __builtin_nontemporal_store(w, as_global(reinterpret_cast<u32x4*>(p)));
    else
        *as_global(reinterpret_cast<u32x4*>(p)) = w;
}

// One row into a lane's state.  w[0] is the row's first dword (the highest power).  J counts the
// rows folded since the register rotation was last at zero: physical register row p holds
// logical row (p + J) mod NE.  The dwords that leave the top are XORed into the tap positions
// of the sparse generator multiple F (fold_taps.h).
template <class F, int JJ>
__device__ __forceinline__ void fold_row(uint32_t (&S)[F::NE][F::NF], const uint32_t (&w)[F::NF])
{
    constexpr int NE = F::NE, NF = F::NF, J = JJ % NE;
    constexpr int top = (NE - 1 - J + NE) % NE;  // logical row NE-1 before the shift
    uint32_t t[NF];
    static_for<NF>([&](auto f) { t[f] = S[top][f]; });
    static_for<NF>([&](auto f) { S[top][f] = w[NF - 1 - f]; });  // becomes logical row 0
    static_for<NF>([&](auto f) {
        static_for<F::NTAP>([&](auto k) {
            constexpr int e = F::TAP_E[f][k];
            constexpr int c = F::TAP_F[f][k];
            if constexpr (e != 255) {
                constexpr int p = (e - (J + 1) + 2 * NE) % NE;
                S[p][c] ^= t[f];
            }
        });
    });
}

// After K rows folded with J = 0..K-1 the physical register rows lag the logical ones by K;
// moving them back makes J = 0 valid again (physical row q takes what physical row q - K held).
template <class F, int K>
__device__ __forceinline__ void rotate_state(uint32_t (&S)[F::NE][F::NF])
{
    constexpr int NE = F::NE, NF = F::NF;
    uint32_t old[NE][NF];
    static_for<NE>([&](auto e) { static_for<NF>([&](auto f) { old[e][f] = S[e][f]; }); });
    static_for<NE>([&](auto q) {
        static_for<NF>([&](auto f) { S[q][f] = old[(q - K % NE + NE) % NE][f]; });
    });
}

// Multiply by a fixed power of x with four byte tables (LDS).
__device__ __forceinline__ uint32_t mul_tab(const uint32_t* tab, uint32_t a)
{
    return tab[a & 0xFFu] ^ tab[256 + ((a >> 8) & 0xFFu)] ^ tab[512 + ((a >> 16) & 0xFFu)] ^
           tab[768 + (a >> 24)];
}

// State of all lanes -> R / x^32, where R is the CRC register (run from 0) of the rows folded so
// far; the factor x^32 that every register carries is applied once per chunk by the combine
// step.  The result is valid in every lane.  tab: byte tables of x^(8*ROW_BYTES);
// lane_c = x^(8 * (ROW_BYTES/64) * (63 - lane)): lane l sits 63 - l lane widths before the end of
// a row.
template <class F>
__device__ __forceinline__ uint32_t reduce_state(const uint32_t (&S)[F::NE][F::NF],
                                                 const uint32_t* tab, uint32_t lane_c)
{
    constexpr int NE = F::NE, NF = F::NF;
    uint32_t acc[NF];
    static_for<NF>([&](auto f) { acc[f] = 0; });
    static_for<NE>([&](auto i) {
        constexpr int e = NE - 1 - i;
        static_for<NF>([&](auto f) { acc[f] = mul_tab(tab, acc[f]) ^ S[e][f]; });
    });
    uint32_t v = acc[NF - 1];
    static_for<NF - 1>([&](auto i) { v = gf2_mul_const<kX32>(v) ^ acc[NF - 2 - i]; });
    v = gf2_mul(v, lane_c);
#pragma unroll
    for (int l = 0; l < 6; l++) v ^= __shfl_xor(v, 1 << l, kWaveSize);
    return v;
}

}  // namespace ffsnap
