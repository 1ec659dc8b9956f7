"""Polynomial arithmetic over GF(2) with Python integers: an independent formulation used to
pin the oracle's CRC (bit i of an int is the coefficient of x^i)."""

POLY = 0x11EDC6F41  # x^32 + ... + 1, the Castagnoli generator, normal (non-reflected) form


def polymod(a, p=POLY):
    dp = p.bit_length() - 1
    while a.bit_length() - 1 >= dp:
        a ^= p << (a.bit_length() - 1 - dp)
    return a


def polymulmod(a, b, p=POLY):
    r = 0
    while b:
        if b & 1:
            r ^= a
        a <<= 1
        b >>= 1
    return polymod(r, p)


def polypowx(e, p=POLY):
    """x^e mod p by square and multiply."""
    r, base = 1, 2
    while e:
        if e & 1:
            r = polymulmod(r, base, p)
        base = polymulmod(base, base, p)
        e >>= 1
    return r


def reflect(v, bits):
    return int(format(v, "0%db" % bits)[::-1], 2) if bits else 0


def message_poly(data):
    """Message as a polynomial: first byte highest, and within a byte bit 0 highest (reflected
    input), so the byte string is read as one long bit-reversed number."""
    m = 0
    for b in bytes(data):
        m = (m << 8) | reflect(b, 8)
    return m


def crc32c_by_division(data):
    """CRC32C from the textbook definition: remainder of M(x)*x^32 with the first 32 message
    bits complemented (the all-ones preset), then complemented and bit-reflected."""
    data = bytes(data)
    n = len(data) * 8
    m = message_poly(data) << 32
    m ^= 0xFFFFFFFF << n            # preset 0xFFFFFFFF == complement the first 32 bits of M*x^32
    return reflect(polymod(m) ^ 0xFFFFFFFF, 32)
