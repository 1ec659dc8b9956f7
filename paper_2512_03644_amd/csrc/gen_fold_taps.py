#!/usr/bin/env python3
"""Writes fold_taps.h: sparse multiples of the CRC32C generator used by the folding kernels.

A wavefront reads a row of ROW bytes per step, lane l taking F consecutive dwords at byte
16*l (F = 4) -- so the dwords one lane sees are ROW/4 = S dword positions apart from row to row.
Writing y = x^32, the lane's part of the message is a polynomial in y whose exponents have the
form S*e + f (e = row counted from the end, f = 0..F-1).  Reducing it needs, for every f, one
multiple of the generator P(x) of the form

    y^(S*NE + f)  +  sum_k  y^(S*e_k + f_k)          (e_k < NE, f_k < F, few terms)

i.e. a congruence  y^(S*NE+f) = sum_k y^(S*e_k+f_k)  (mod P).  With it the lane keeps NE*F
dwords of state; each new row shifts the state up by one row and the F dwords that fall off the
top are XORed into the tap positions (e_k, f_k).  Everything is exact GF(2) algebra, so the
folded state is congruent to the message modulo P.  Because x+1 divides P every multiple has an
even number of terms, so the tap count is odd.

The search is a meet-in-the-middle over the NE*F candidate exponents; the lexicographically
smallest solution is taken so that the output is reproducible.
"""
import itertools
import os
import sys

import numpy as np

POLY = 0x11EDC6F41


def polymod(a):
    while a.bit_length() > 32:
        a ^= POLY << (a.bit_length() - 33)
    return a


def polymul(a, b):
    r = 0
    while b:
        if b & 1:
            r ^= a
        a <<= 1
        b >>= 1
    return polymod(r)


def xpow(e):
    r, base = 1, 2
    while e:
        if e & 1:
            r = polymul(r, base)
        base = polymul(base, base)
        e >>= 1
    return r


def solve_min_weight(S, F, NE):
    """For a small surplus of candidates over the 32 dimensions of the residue space: solve the
    linear system by Gaussian elimination, then walk the whole solution set (one particular
    solution plus the null space) and keep the representation with the fewest terms."""
    cand = [S * e + f for e in range(NE) for f in range(F)]
    n = len(cand)
    vecs = [xpow(32 * E) for E in cand]
    basis = {}     # highest bit -> (value, mask of candidates)
    null = []      # masks of candidate subsets that XOR to zero
    for i, v in enumerate(vecs):
        m = 1 << i
        while v:
            hb = v.bit_length() - 1
            if hb in basis:
                v ^= basis[hb][0]
                m ^= basis[hb][1]
            else:
                basis[hb] = (v, m)
                break
        if not v:
            null.append(m)
    assert len(null) <= 20, "too many candidates for exhaustive enumeration"
    out = []
    for f in range(F):
        v, m = xpow(32 * (S * NE + f)), 0
        while v:
            hb = v.bit_length() - 1
            if hb not in basis:
                raise SystemExit("target outside the span for S=%d F=%d NE=%d f=%d" % (S, F, NE, f))
            v ^= basis[hb][0]
            m ^= basis[hb][1]
        best = None
        for k in range(1 << len(null)):
            mm = m
            for j, nm in enumerate(null):
                if (k >> j) & 1:
                    mm ^= nm
            key = (bin(mm).count("1"), mm)
            if best is None or key < best:
                best = key
        taps = [i for i in range(n) if (best[1] >> i) & 1]
        acc = xpow(32 * (S * NE + f))
        for i in taps:
            acc ^= vecs[i]
        assert acc == 0
        out.append([(cand[i] // S, cand[i] % S) for i in taps])
    return out


def search(S, F, NE, ntaps):
    if ntaps == 0:
        return solve_min_weight(S, F, NE)
    cand = [S * e + f for e in range(NE) for f in range(F)]
    r = np.array([xpow(32 * E) for E in cand], dtype=np.uint64)
    n = len(cand)
    ka = ntaps // 2
    kb = ntaps - ka

    def subsets(k):
        idx = np.array(list(itertools.combinations(range(n), k)), dtype=np.int32)
        x = np.zeros(len(idx), dtype=np.uint64)
        for c in range(k):
            x ^= r[idx[:, c]]
        return idx, x

    ia, xa = subsets(ka)
    ib, xb = subsets(kb)
    order = np.argsort(xa, kind="stable")
    xs = xa[order]
    out = []
    for f in range(F):
        target = np.uint64(xpow(32 * (S * NE + f)))
        q = xb ^ target
        pos = np.searchsorted(xs, q)
        pos[pos >= len(xs)] = len(xs) - 1
        sols = set()
        for h in np.nonzero(xs[pos] == q)[0]:
            p = pos[h]
            while p < len(xs) and xs[p] == q[h]:
                s = set(ia[order[p]].tolist()) | set(ib[h].tolist())
                if len(s) == ntaps:
                    sols.add(tuple(sorted(s)))
                p += 1
        if not sols:
            raise SystemExit("no %d-tap relation for S=%d F=%d NE=%d f=%d" % (ntaps, S, F, NE, f))
        best = min(sols)
        # check the congruence once more with plain integer arithmetic
        acc = xpow(32 * (S * NE + f))
        for i in best:
            acc ^= xpow(32 * cand[i])
        assert acc == 0
        out.append([(cand[i] // S, cand[i] % S) for i in best])
    return out


SETS = [
    # name, row bytes, dwords per lane, NE, taps
    ("Fold16x16", 1024, 4, 16, 9),
    # 0 = fewest terms found by exhaustive walk of the solution set (few candidates, small state)
    ("Fold16x10", 1024, 4, 10, 0),
    ("Fold8x20", 512, 2, 20, 0),
]


def emit(path):
    lines = ["// Generated by gen_fold_taps.py -- do not edit.  Sparse multiples of the CRC32C generator;",
             "// see the generator's docstring for the algebra.  TAP_E/TAP_F[f][k]: the dword that",
             "// leaves the top of column f is XORed into state position (row TAP_E, column TAP_F).",
             "#pragma once", "", "namespace ffsnap {", ""]
    for name, row, F, NE, nt in SETS:
        S = row // 4
        taps = search(S, F, NE, nt)
        nt = max(len(t) for t in taps)
        used = [len(t) for t in taps]
        taps = [t + [(255, 255)] * (nt - len(t)) for t in taps]  # 255 = unused slot
        lines += ["struct %s {" % name,
                  "    static constexpr int ROW_BYTES = %d;  // bytes one wavefront reads per step" % row,
                  "    static constexpr int STRIDE = %d;     // dword distance between a lane's rows" % S,
                  "    static constexpr int NF = %d;         // dwords per lane per row" % F,
                  "    static constexpr int NE = %d;         // rows of state" % NE,
                  "    static constexpr int NTAP = %d;       // slots per column (255 = unused)" % nt]
        for nm, sel in (("TAP_E", 0), ("TAP_F", 1)):
            rows = ["{" + ", ".join(str(t[sel]) for t in taps[f]) + "}" for f in range(F)]
            lines.append("    static constexpr unsigned char %s[NF][NTAP] = {%s};" % (nm, ", ".join(rows)))
        lines += ["};", ""]
    lines += ["}  // namespace ffsnap", ""]
    with open(path, "w") as fh:
        fh.write("\n".join(lines))


if __name__ == "__main__":
    emit(sys.argv[1] if len(sys.argv) > 1 else
         os.path.join(os.path.dirname(os.path.abspath(__file__)), "fold_taps.h"))
