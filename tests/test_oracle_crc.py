"""Pins for the oracle's CRC32C: published vectors, polynomial long division, brute force."""
import os

import numpy as np
import pytest

from gf2ref import crc32c_by_division, polymulmod, polypowx, reflect

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "crc32c_vectors.txt")


def _vectors():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        crc, kind, *args = line.split()
        if kind == "ascii":
            data = args[0].encode()
        elif kind == "fill":
            data = bytes([int(args[1], 16)]) * int(args[0])
        elif kind == "incr":
            data = bytes(range(int(args[0])))
        elif kind == "decr":
            data = bytes(reversed(range(int(args[0]))))
        else:
            raise ValueError(kind)
        out.append((int(crc, 16), data))
    return out


def _u8(b):
    return np.frombuffer(bytes(b), dtype=np.uint8)


def test_published_vectors(oracle):
    vecs = _vectors()
    assert len(vecs) >= 7
    for crc, data in vecs:
        assert oracle.crc32c_bitwise(_u8(data)) == crc
        assert oracle.crc32c(_u8(data)) == crc
        assert crc32c_by_division(data) == crc


def test_bitwise_matches_polynomial_division(oracle):
    rng = np.random.default_rng(1)
    for n in list(range(0, 70)) + [127, 128, 129, 255, 256, 300, 1000]:
        data = rng.integers(0, 256, size=n, dtype=np.uint8)
        assert oracle.crc32c_bitwise(data) == crc32c_by_division(data.tobytes())


def test_table_matches_bitwise_every_length_and_alignment(oracle):
    rng = np.random.default_rng(2)
    base = rng.integers(0, 256, size=4096 + 64, dtype=np.uint8)
    for n in range(0, 4097):
        a = int(rng.integers(0, 64))
        piece = base[a:a + n]
        assert oracle.crc32c(piece) == oracle.crc32c_bitwise(piece), (n, a)


def test_shift_is_multiplication_by_x_power(oracle):
    # shift(c, n) == c(x) * x^(8n) mod P on the bit-reflected register contents
    rng = np.random.default_rng(3)
    for n in [0, 1, 2, 3, 4, 15, 16, 17, 1024, 4096, 65536, 1 << 20]:
        c = int(rng.integers(0, 1 << 32))
        want = reflect(polymulmod(reflect(c, 32), polypowx(8 * n)), 32)
        assert oracle.crc_shift(c, n) == want, n


def test_shift_additive_and_linear(oracle):
    rng = np.random.default_rng(4)
    for _ in range(50):
        c, d = (int(x) for x in rng.integers(0, 1 << 32, size=2))
        a, b = (int(x) for x in rng.integers(0, 3000, size=2))
        assert oracle.crc_shift(c, a + b) == oracle.crc_shift(oracle.crc_shift(c, a), b)
        assert oracle.crc_shift(c ^ d, a) == oracle.crc_shift(c, a) ^ oracle.crc_shift(d, a)
    assert oracle.crc_shift(0, 12345) == 0


def test_combine_identity_brute_force(oracle):
    rng = np.random.default_rng(5)
    for _ in range(200):
        la, lb = (int(x) for x in rng.integers(0, 600, size=2))
        a = rng.integers(0, 256, size=la, dtype=np.uint8)
        b = rng.integers(0, 256, size=lb, dtype=np.uint8)
        ab = np.concatenate([a, b])
        # raw register (no preset, no complement): exact, no correction term
        ra, rb = oracle.crc_reg(0, a), oracle.crc_reg(0, b)
        assert oracle.crc_shift(ra, lb) ^ rb == oracle.crc_reg(0, ab)
        # standard CRC written through the raw register:
        #   crc(D) = reg0(D) ^ shift(0xFFFFFFFF, |D|) ^ 0xFFFFFFFF
        assert oracle.crc32c(ab) == oracle.crc_reg(0, ab) ^ \
            oracle.crc_shift(0xFFFFFFFF, la + lb) ^ 0xFFFFFFFF


def test_combine_standard_crc(oracle):
    # crc(A||B) = shift(crc(A), |B|) ^ crc(B) ^ shift(0, ..) -- for the standard CRC the preset
    # of B and the complement of A cancel: shift(crc(A) ^ 0xFFFFFFFF ^ 0xFFFFFFFF ...).  Check the
    # form the oracle exports against direct evaluation.
    rng = np.random.default_rng(6)
    for _ in range(200):
        la, lb = (int(x) for x in rng.integers(0, 600, size=2))
        a = rng.integers(0, 256, size=la, dtype=np.uint8)
        b = rng.integers(0, 256, size=lb, dtype=np.uint8)
        want = oracle.crc32c(np.concatenate([a, b]))
        # state after A is crc(A)^0xFFFFFFFF; B starts from it instead of from 0xFFFFFFFF
        got = oracle.crc_shift(oracle.crc32c(a) ^ 0xFFFFFFFF ^ 0xFFFFFFFF, lb) ^ oracle.crc32c(b)
        assert got == want
        assert oracle.crc32c_combine(oracle.crc32c(a), oracle.crc32c(b), lb) == want


def test_every_single_bit_flip_changes_the_crc(oracle):
    rng = np.random.default_rng(7)
    data = rng.integers(0, 256, size=96, dtype=np.uint8)
    ref = oracle.crc32c(data)
    for i in range(data.size):
        for bit in range(8):
            d = data.copy()
            d[i] ^= 1 << bit
            assert oracle.crc32c(d) != ref
    big = rng.integers(0, 256, size=1 << 16, dtype=np.uint8)
    ref = oracle.crc32c(big)
    for _ in range(64):
        d = big.copy()
        d[int(rng.integers(0, big.size))] ^= 1 << int(rng.integers(0, 8))
        assert oracle.crc32c(d) != ref


def test_zero_prefix_does_not_change_the_raw_register(oracle):
    rng = np.random.default_rng(8)
    a = rng.integers(0, 256, size=100, dtype=np.uint8)
    z = np.zeros(37, dtype=np.uint8)
    assert oracle.crc_reg(0, np.concatenate([z, a])) == oracle.crc_reg(0, a)
