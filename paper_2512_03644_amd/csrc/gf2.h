// GF(2) polynomial arithmetic modulo the CRC32C generator, in the bit-reflected representation
// the CRC uses: a 32-bit word holds a polynomial of degree < 32 with bit 31 = x^0 and
// bit 0 = x^31.  A little-endian dword read from the byte stream already has this form (first
// byte, lowest bit = highest power), so stream data and CRC registers mix with plain XOR.
//
// With this convention the register of a CRC run from 0 over a message M (no preset, no final
// complement) is M(x) * x^32 mod P, and appending n bytes multiplies a register by x^(8n).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FF_HD __host__ __device__ constexpr inline
#else
#define FF_HD constexpr inline
#endif

namespace ffsnap {

constexpr uint32_t kPolyReflected = 0x82F63B78u;  // 0x1EDC6F41 bit-reversed
constexpr uint32_t kOne = 0x80000000u;            // the polynomial 1

// a * x mod P
FF_HD uint32_t gf2_mulx(uint32_t a) { return (a >> 1) ^ ((a & 1u) ? kPolyReflected : 0u); }

// a * b mod P
FF_HD uint32_t gf2_mul(uint32_t a, uint32_t b)
{
    uint32_t p = 0;
    for (int i = 0; i < 32; i++) {
        p ^= (a & 0x80000000u) ? b : 0u;  // coefficient of x^i in a
        a <<= 1;
        b = gf2_mulx(b);
    }
    return p;
}

// a * C mod P for a multiplier known at compile time: the powers C*x^i fold to literals, which
// leaves a bit test, an AND and an XOR per bit.
template <uint32_t C>
FF_HD uint32_t gf2_mul_const(uint32_t a)
{
    uint32_t p = 0, b = C;
    for (int i = 0; i < 32; i++) {
        p ^= (a & 0x80000000u) ? b : 0u;
        a <<= 1;
        b = gf2_mulx(b);
    }
    return p;
}

// x^32 mod P is the generator without its leading term.
constexpr uint32_t kX32 = kPolyReflected;

// x^n mod P
constexpr inline uint32_t gf2_xpow(uint64_t n)
{
    uint32_t r = kOne, base = kOne >> 1;  // 1, x
    while (n) {
        if (n & 1) r = gf2_mul(r, base);
        base = gf2_mul(base, base);
        n >>= 1;
    }
    return r;
}

// CRC32C of a host buffer, bit by bit (used for the layout id only).
inline uint32_t crc32c_host(const void* data, uint64_t n)
{
    const unsigned char* p = static_cast<const unsigned char*>(data);
    uint32_t c = 0xFFFFFFFFu;
    for (uint64_t i = 0; i < n; i++) {
        c ^= p[i];
        for (int k = 0; k < 8; k++) c = gf2_mulx(c);
    }
    return ~c;
}

// What the preset and the final complement add to the register of an n-byte message:
// crc(M) = reg0(M) ^ crc_affine_term(n).
inline uint32_t crc_affine_term(uint64_t nbytes)
{
    return gf2_mul(0xFFFFFFFFu, gf2_xpow(8 * nbytes)) ^ 0xFFFFFFFFu;
}

}  // namespace ffsnap
