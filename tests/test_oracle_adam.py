"""Pins for the oracle's AdamW step: torch.optim.AdamW in float64 (library routine), closed-form
special cases, torch's bf16 cast for the rounding."""
import numpy as np
import pytest
import torch

HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1000)


def _f32(x):
    return float(np.float32(x))


def _draw(n, seed):
    rng = np.random.default_rng(seed)
    master = rng.normal(0, 0.02, n).astype(np.float32)
    m = rng.normal(0, 1e-3, n).astype(np.float32)
    v = (rng.normal(0, 1e-3, n).astype(np.float32)) ** 2
    g32 = rng.normal(0, 1e-3, n).astype(np.float32)
    g16 = torch.from_numpy(g32).to(torch.bfloat16)
    return master, m, v, g16


def _bits(t16):
    return t16.view(torch.int16).numpy().view(np.uint16).copy()


def _torch_adamw_f64(master, m, v, g, hp):
    p = torch.tensor(master, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                            weight_decay=hp["weight_decay"])
    p.grad = torch.tensor(g, dtype=torch.float64)
    opt.step()  # materialise state, then overwrite it and redo the step from the given state
    st = opt.state[p]
    with torch.no_grad():
        p.copy_(torch.tensor(master, dtype=torch.float64))
        st["exp_avg"].copy_(torch.tensor(m, dtype=torch.float64))
        st["exp_avg_sq"].copy_(torch.tensor(v, dtype=torch.float64))
        st["step"].fill_(hp["step"] - 1)
    opt.step()
    return (p.detach().numpy(), st["exp_avg"].numpy(), st["exp_avg_sq"].numpy())


@pytest.mark.parametrize("step", [1, 2, 10, 1000])
def test_f64_step_matches_torch_adamw(oracle, step):
    hp = dict(HP, step=step)
    hp64 = {k: (_f32(x) if k != "step" else x) for k, x in hp.items()}
    master, m, v, g16 = _draw(257, 21 + step)
    g = g16.to(torch.float64).numpy()
    M, A, B = (x.astype(np.float64) for x in (master, m, v))
    want = _torch_adamw_f64(M, A, B, g, hp64)
    oracle.adam_f64(g.copy(), M, A, B, **hp64)
    for got, w in zip((M, A, B), want):
        np.testing.assert_allclose(got, w, rtol=1e-12, atol=1e-300)


@pytest.mark.parametrize("step", [1, 7, 1000])
def test_f32_step_close_to_f64_step(oracle, step):
    hp = dict(HP, step=step)
    master, m, v, g16 = _draw(4096, 31 + step)
    w16 = np.zeros(master.size, dtype=np.uint16)
    g = g16.to(torch.float64).numpy()
    M, A, B = (x.astype(np.float64) for x in (master, m, v))
    hp64 = {k: (_f32(x) if k != "step" else x) for k, x in hp.items()}
    oracle.adam_f64(g.copy(), M, A, B, **hp64)
    m0, v0, p0 = m.copy(), v.copy(), master.copy()
    oracle.adam_f32(_bits(g16), master, m, v, w16, **hp)
    u = 2.0 ** -24
    # m' = b1*m + (1-b1)*g can cancel: bound by the magnitudes of its terms
    bound_m = 4 * u * (np.abs(0.9 * m0.astype(np.float64)) + np.abs(0.1 * g)) + 1e-45
    assert np.all(np.abs(m - A) <= bound_m)
    np.testing.assert_allclose(v, B, rtol=8 * u, atol=1e-45)
    # update term: |step_size*m'/d| amplifies m' error by 1/d
    d = np.sqrt(B) / np.sqrt(1 - hp64["beta2"] ** step) + hp64["eps"]
    ss = hp64["lr"] / (1 - hp64["beta1"] ** step)
    bound_p = 8 * u * (np.abs(p0) + ss * np.abs(A) / d) + ss * bound_m / d
    assert np.all(np.abs(master - M) <= bound_p)


def test_special_cases(oracle):
    n = 1000
    master, m, v, g16 = _draw(n, 41)
    w16 = np.zeros(n, dtype=np.uint16)
    zero = np.zeros(n, dtype=np.uint16)
    # g = 0, no decay: moments decay geometrically, each one fp32 product
    p, a, b = master.copy(), m.copy(), v.copy()
    oracle.adam_f32(zero, p, a, b, w16, **dict(HP, weight_decay=0.0))
    assert np.array_equal(a, np.float32(0.9) * m)
    assert np.array_equal(b, np.float32(0.95) * v)
    # lr = 0: parameters unchanged whatever the moments
    p, a, b = master.copy(), m.copy(), v.copy()
    oracle.adam_f32(_bits(g16), p, a, b, w16, **dict(HP, lr=0.0))
    assert np.array_equal(p, master)
    # first step from zero moments, no decay: sign-like update  -lr * g / (|g| + eps)
    p = master.copy()
    a = np.zeros(n, dtype=np.float32)
    b = np.zeros(n, dtype=np.float32)
    hp = dict(HP, weight_decay=0.0, step=1)
    oracle.adam_f32(_bits(g16), p, a, b, w16, **hp)
    g = g16.to(torch.float64).numpy()
    want = master.astype(np.float64) - _f32(hp["lr"]) * g / (np.abs(g) + _f32(hp["eps"]))
    np.testing.assert_allclose(p, want, rtol=0, atol=3e-4 * 1e-5 + 1e-9)
    # decay only (g = 0, m = 0): master shrinks by exactly fp32(1 - lr*wd)
    p = master.copy()
    a = np.zeros(n, dtype=np.float32)
    b = np.ones(n, dtype=np.float32)
    oracle.adam_f32(zero, p, a, b, w16, **HP)
    decay = np.float32(1.0 - np.float64(np.float32(3e-4)) * np.float64(np.float32(0.1)))
    assert np.array_equal(p, master * decay)


@pytest.mark.parametrize("fp16", [False, True])
def test_nan_results_take_the_canonical_form(oracle, fp16):
    """A new master, m or v that is NaN is stored as 0x7FC00000 whatever the sign and payload of
    the NaN that went in or that the arithmetic produced, the 16-bit weight is rounded from that
    (bf16 0x7FC0, fp16 0x7E00); NaN-ness itself is the arithmetic's (checked against float64),
    and every other element is what the step gives without the rule."""
    n = 64
    master, m, v, g16 = _draw(n, 5)
    u = lambda bits: np.array([bits], dtype=np.uint32).view(np.float32)[0]
    # NaNs of either sign with payloads, in each input; inf - inf and 0 * inf produced inside
    m[0], m[1] = u(0x7FC12345), u(0xFFFFFFFF)          # quiet +, quiet - with full payload
    v[2] = u(0xFF800001)                               # signalling, negative
    master[3], master[4] = u(0xFFC00000), u(0x7F800123)
    v[5] = -1.0                                        # sqrt of a negative number
    master[6], m[6] = np.float32(np.inf), np.float32(np.inf)      # inf - inf in the last line
    gbits = _bits(g16)
    g_f32 = g16.to(torch.float32).numpy()
    if fp16:
        gbits = torch.from_numpy(g_f32).to(torch.float16).view(torch.int16).numpy().view(np.uint16).copy()
        g_f32 = torch.from_numpy(gbits.view(np.int16)).view(torch.float16).to(torch.float32).numpy()
        gbits[7] = 0xFE01                              # a NaN gradient
        g_f32[7] = np.nan
    ref = [x.copy() for x in (master, m, v)]
    w16 = np.zeros(n, dtype=np.uint16)
    if fp16:
        oracle.adam_f32_f16(gbits, 1.0, master, m, v, w16, **HP)
    else:
        oracle.adam_f32(gbits, master, m, v, w16, **HP)
    # NaN-ness per element from the same formulas in float64 (numpy)
    hp = {k: (float(np.float32(x)) if k != "step" else x) for k, x in HP.items()}
    with np.errstate(all="ignore"):
        P, M, V = (x.astype(np.float64) for x in ref)
        g = g_f32.astype(np.float64)
        m1 = hp["beta1"] * M + (1 - hp["beta1"]) * g
        v1 = hp["beta2"] * V + (1 - hp["beta2"]) * g * g
        d = np.sqrt(v1) / np.sqrt(1 - hp["beta2"] ** hp["step"]) + hp["eps"]
        p1 = P * (1 - hp["lr"] * hp["weight_decay"]) - hp["lr"] / (1 - hp["beta1"] ** hp["step"]) * (m1 / d)
    n_nan = 0
    for got, want in ((master, p1), (m, m1), (v, v1)):
        bits = got.view(np.uint32)
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got), nan)
        assert bool((bits[nan] == 0x7FC00000).all())
        n_nan += int(nan.sum())
    assert n_nan >= (12 if fp16 else 9)
    assert bool((w16[np.isnan(p1)] == (0x7E00 if fp16 else 0x7FC0)).all())
    # the elements without any NaN: the same values as a run whose NaN sources are replaced
    clean = ~(np.isnan(p1) | np.isnan(m1) | np.isnan(v1))
    assert clean.sum() >= n - 8
    a, b, c = (x.copy() for x in ref)
    for arr in (a, b, c):
        arr[~clean] = 1.0
    gb = gbits.copy()
    gb[~clean] = 0
    w2 = np.zeros(n, dtype=np.uint16)
    if fp16:
        oracle.adam_f32_f16(gb, 1.0, a, b, c, w2, **HP)
    else:
        oracle.adam_f32(gb, a, b, c, w2, **HP)
    for got, other in ((master, a), (m, b), (v, c)):
        assert np.array_equal(got.view(np.uint32)[clean], other.view(np.uint32)[clean])
    assert np.array_equal(w16[clean], w2[clean])


def test_bf16_weight_is_rne_of_the_new_master(oracle):
    n = 5000
    master, m, v, g16 = _draw(n, 51)
    w16 = np.zeros(n, dtype=np.uint16)
    oracle.adam_f32(_bits(g16), master, m, v, w16, **HP)
    assert np.array_equal(w16, _bits(torch.from_numpy(master).to(torch.bfloat16)))


def test_bf16_rounding_cases(oracle):
    rng = np.random.default_rng(61)
    bits = rng.integers(0, 1 << 32, size=20000, dtype=np.uint64).astype(np.uint32)
    # ties, near-ties, infinities, denormals, max finite (rounds to infinity)
    extra = np.array([0x3F808000, 0x3F818000, 0x3F807FFF, 0x3F808001, 0x7F800000, 0xFF800000,
                      0x00000001, 0x00008000, 0x00018000, 0x7F7FFFFF, 0x80000000, 0],
                     dtype=np.uint32)
    bits = np.concatenate([bits, extra])
    f = bits.view(np.float32)
    finite_or_inf = ~np.isnan(f)
    want = _bits(torch.from_numpy(f.copy()).to(torch.bfloat16))
    got = np.array([oracle.f32_to_bf16(float(x)) for x in f[finite_or_inf]], dtype=np.uint16)
    assert np.array_equal(got, want[finite_or_inf])
    # NaN stays NaN, keeps its sign, never becomes infinity
    for u in (0x7F800001, 0x7FC00000, 0xFF800001, 0x7FFFFFFF, 0x7F80FFFF):
        h = oracle.lib().orc_f32_to_bf16(np.array([u], dtype=np.uint32).view(np.float32)[0])
        assert (h & 0x7F80) == 0x7F80 and (h & 0x007F) != 0 and (h >> 15) == (u >> 31)


# ---- fp16 variant: conversions and the loss-scaled step ------------------------------------------

def test_f16_decode_every_value(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.f16_to_f32(bits)
    want = bits.view(np.float16).astype(np.float32)        # numpy's IEEE conversion, exact
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])
    # closed form of a few values
    for h, x in [(0x3C00, 1.0), (0xC000, -2.0), (0x7BFF, 65504.0), (0x0001, 2.0 ** -24),
                 (0x0400, 2.0 ** -14), (0x03FF, 1023 * 2.0 ** -24), (0x8000, -0.0)]:
        r = oracle.f16_to_f32(np.array([h], dtype=np.uint16))[0]
        assert r == np.float32(x) and np.signbit(r) == np.signbit(np.float32(x))
    assert np.isposinf(oracle.f16_to_f32(np.array([0x7C00], dtype=np.uint16))[0])


def test_f16_encode_round_trip_ties_and_limits(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16).astype(np.float32)
    finite = ~np.isnan(vals)
    # every fp16 value survives the round trip
    assert np.array_equal(oracle.f32_to_f16(vals[finite]), bits[finite])
    # every midpoint between neighbouring positive fp16 values (exact in fp32) goes to the even one
    lo = np.arange(0, 0x7BFF, dtype=np.uint16)
    a = lo.view(np.float16).astype(np.float64)
    b = (lo + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((a + b) / 2).astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), (a + b) / 2)
    want = np.where(lo % 2 == 0, lo, lo + 1).astype(np.uint16)
    assert np.array_equal(oracle.f32_to_f16(mid), want)
    assert np.array_equal(oracle.f32_to_f16(-mid), want | 0x8000)
    # one fp32 step to either side of a midpoint goes to the nearer neighbour
    up = np.nextafter(mid, np.float32(np.inf))
    dn = np.nextafter(mid, np.float32(-np.inf))
    assert np.array_equal(oracle.f32_to_f16(up), lo + 1)
    assert np.array_equal(oracle.f32_to_f16(dn[1:]), lo[1:])
    # limits: the largest value, the overflow threshold 65520, underflow to zero at 2^-25
    one = lambda x: int(oracle.f32_to_f16(np.array([x], dtype=np.float32))[0])
    assert one(65504.0) == 0x7BFF and one(np.nextafter(np.float32(65520), np.float32(0))) == 0x7BFF
    assert one(65520.0) == 0x7C00 and one(1e9) == 0x7C00 and one(-1e9) == 0xFC00
    assert one(np.inf) == 0x7C00 and one(-np.inf) == 0xFC00
    assert one(2.0 ** -25) == 0 and one(np.nextafter(np.float32(2.0 ** -25), np.float32(1))) == 1
    assert one(-(2.0 ** -25)) == 0x8000 and one(0.0) == 0 and one(-0.0) == 0x8000
    assert one(1e-30) == 0 and one(2.0 ** -24) == 1 and one(2.0 ** -14) == 0x0400
    # NaN: quiet, sign and top payload bits kept
    q = np.array([0x7FC00000, 0xFFC00000, 0x7F800001, 0x7FA12345], dtype=np.uint32).view(np.float32)
    got = oracle.f32_to_f16(q)
    assert list(got) == [0x7E00, 0xFE00, 0x7E00, 0x7E00 | (0x212345 >> 13)]


def test_f16_encode_matches_numpy_on_random_values(oracle):
    rng = np.random.default_rng(99)
    x = np.concatenate([rng.normal(0, 1, 200000), rng.normal(0, 1e-5, 100000),
                        rng.normal(0, 3e4, 100000),
                        np.exp(rng.uniform(-20, 12, 200000)) * rng.choice([-1, 1], 200000)])
    x = x.astype(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)          # library routine: IEEE RNE
    assert np.array_equal(oracle.f32_to_f16(x), want)


def _draw_f16(n, seed, scale):
    rng = np.random.default_rng(seed)
    master = rng.normal(0, 0.02, n).astype(np.float32)
    m = rng.normal(0, 1e-3, n).astype(np.float32)
    v = (rng.normal(0, 1e-3, n).astype(np.float32)) ** 2
    g = (rng.normal(0, 1e-3, n) * scale).astype(np.float16)  # gradient of the scaled loss
    return master, m, v, g.view(np.uint16).copy()


@pytest.mark.parametrize("step,scale", [(1, 1.0), (7, 1024.0), (1000, 65536.0)])
def test_f16_step_close_to_f64_step(oracle, step, scale):
    hp = dict(HP, step=step)
    n = 4096
    master, m, v, gb = _draw_f16(n, 41 + step, scale)
    inv = float(np.float32(1.0 / scale))
    g64 = gb.view(np.float16).astype(np.float64) * inv
    M, A, B = (x.astype(np.float64) for x in (master, m, v))
    hp64 = {k: (_f32(x) if k != "step" else x) for k, x in hp.items()}
    oracle.adam_f64(g64.copy(), M, A, B, **hp64)
    w16 = np.zeros(n, dtype=np.uint16)
    p, a, b = master.copy(), m.copy(), v.copy()
    bad = oracle.adam_f32_f16(gb, inv, p, a, b, w16, **hp)
    assert bad == 0
    u = 2.0 ** -24
    # same cancellation-aware bounds as for the bf16 step; the unscaling adds one rounding of g
    bound_m = 6 * u * (np.abs(0.9 * m.astype(np.float64)) + np.abs(0.1 * g64)) + 1e-45
    assert np.all(np.abs(a - A) <= bound_m)
    np.testing.assert_allclose(b, B, rtol=12 * u, atol=1e-45)
    d = np.sqrt(B) / np.sqrt(1 - hp64["beta2"] ** step) + hp64["eps"]
    ss = hp64["lr"] / (1 - hp64["beta1"] ** step)
    bound_p = 8 * u * (np.abs(master) + ss * np.abs(A) / d) + ss * bound_m / d
    assert np.all(np.abs(p - M) <= bound_p)
    # the fp16 weights are the rounding of the new master (checked with numpy's conversion)
    assert np.array_equal(w16, p.astype(np.float16).view(np.uint16))


def test_f16_step_equals_bf16_step_on_shared_values(oracle):
    """Gradients that both 16-bit formats represent exactly (small powers of two times small
    integers) with a loss scale of one: master, m and v must come out bit-identical to the bf16
    step's, whose arithmetic is pinned above."""
    rng = np.random.default_rng(5)
    n = 2048
    master, m, v, _ = _draw_f16(n, 77, 1.0)
    g = (rng.integers(-7, 8, n) * 2.0 ** rng.integers(-12, -4, n)).astype(np.float32)
    g_f16 = g.astype(np.float16)
    g_bf16 = torch.from_numpy(g).to(torch.bfloat16)
    assert np.array_equal(g_f16.astype(np.float32), g)
    assert np.array_equal(g_bf16.to(torch.float32).numpy(), g)
    p1, a1, b1 = master.copy(), m.copy(), v.copy()
    p2, a2, b2 = master.copy(), m.copy(), v.copy()
    w1 = np.zeros(n, dtype=np.uint16)
    w2 = np.zeros(n, dtype=np.uint16)
    oracle.adam_f32(_bits(g_bf16), p1, a1, b1, w1, **HP)
    bad = oracle.adam_f32_f16(g_f16.view(np.uint16).copy(), 1.0, p2, a2, b2, w2, **HP)
    assert bad == 0
    for x, y in ((p1, p2), (a1, a2), (b1, b2)):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    # a power-of-two loss scale changes nothing either: g*S is exact in fp16 here, and g*S/S is g
    p3, a3, b3 = master.copy(), m.copy(), v.copy()
    w3 = np.zeros(n, dtype=np.uint16)
    oracle.adam_f32_f16((g * 8).astype(np.float16).view(np.uint16).copy(), 0.125, p3, a3, b3, w3, **HP)
    for x, y in ((p1, p3), (a1, a3), (b1, b3)):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    assert np.array_equal(w2, w3)


def test_f16_step_counts_nonfinite_gradients(oracle):
    n = 1000
    master, m, v, gb = _draw_f16(n, 3, 256.0)
    gb[[5, 17, 900]] = [0x7C00, 0xFC00, 0x7E01]         # +inf, -inf, NaN
    w16 = np.zeros(n, dtype=np.uint16)
    p, a, b = master.copy(), m.copy(), v.copy()
    bad = oracle.adam_f32_f16(gb, 1.0 / 256, p, a, b, w16, **HP)
    assert bad == 3
    ok = np.ones(n, dtype=bool)
    ok[[5, 17, 900]] = False
    assert np.isfinite(p[ok]).all() and np.isfinite(a[ok]).all() and np.isfinite(b[ok]).all()
    assert not np.isfinite(a[5]) and not np.isfinite(a[17]) and np.isnan(a[900])


# ---- the step that reads its state from the previous snapshot ------------------------------------

def _chained_case(seed, numels, half=torch.bfloat16):
    """Parameter groups with a RAW segment in between, the previous state as its own arrays, and
    the previous snapshot built with numpy alone (tight concatenation, zero fill)."""
    rng = np.random.default_rng(seed)
    segs, params, grads, prev_state = [], [], [], []
    for k, n in enumerate(numels):
        master, m, v, g16 = _draw(n, seed + k)
        w_old = _bits(torch.from_numpy(master).to(half))
        prev_state.append((w_old, master, m, v))
        # what the step is given: arrays of the right sizes holding garbage it must not use
        grp = (np.full(n, 0x7FC1, np.uint16), np.full(n, np.nan, np.float32),
               np.full(n, np.nan, np.float32), np.full(n, np.nan, np.float32))
        params.append(grp)
        segs += list(grp)
        grads.append(_bits(g16.to(torch.float32).to(half)))
        if k == 0:
            segs.append(rng.integers(0, 256, 333 * 2, dtype=np.uint8))  # a RAW segment
    return segs, params, grads, prev_state


def _numpy_buffer(arrays, chunk):
    stream = np.concatenate([np.ascontiguousarray(a).view(np.uint8).reshape(-1) for a in arrays])
    n_chunks = -(-stream.size // chunk)
    buf = np.zeros(n_chunks * chunk, np.uint8)
    buf[:stream.size] = stream
    return buf


def test_chained_step_takes_its_state_from_the_previous_snapshot(oracle):
    chunk, numels = 4096, [1000, 3, 4099]
    segs, params, grads, prev_state = _chained_case(7, numels)
    raw = segs[4]
    prev_list = []
    for k, grp in enumerate(prev_state):
        prev_list += list(grp)
        if k == 0:
            prev_list.append(np.zeros_like(raw))  # the RAW bytes of the old snapshot are not used
    prev = _numpy_buffer(prev_list, chunk)
    buf, crcs, bad = oracle.adam_snapshot_chained(prev, params, grads, segs, chunk, HP)
    assert bad == 0
    # expected: the pinned single-tensor step on the old state, laid out with numpy alone
    want = []
    for k, ((w, master, m, v), g) in enumerate(zip(prev_state, grads)):
        master, m, v, w = master.copy(), m.copy(), v.copy(), w.copy()
        oracle.adam_f32(g, master, m, v, w, **HP)
        want += [w, master, m, v]
        if k == 0:
            want.append(raw)
        assert np.array_equal(params[k][0], w)          # the new working weights are handed back
    want_buf = _numpy_buffer(want, chunk)
    assert np.array_equal(buf, want_buf)
    assert [int(c) for c in crcs] == [oracle.crc32c_bitwise(want_buf[i:i + chunk])
                                      for i in range(0, want_buf.size, chunk)]


def test_chained_step_closed_form(oracle):
    # g = 0, lr = 0, wd = 0: master' = master, m' = fl(b1 m), v' = fl(b2 v), w' = bf16(master);
    # distinct m and v at distinct offsets, so a stream read from the wrong place shows
    chunk, numels = 1024, [777, 130]
    segs, params, grads, prev_state = _chained_case(11, numels)
    grads = [np.zeros_like(g) for g in grads]
    hp = dict(HP, lr=0.0, weight_decay=0.0)
    prev_list = []
    for k, grp in enumerate(prev_state):
        prev_list += list(grp)
        if k == 0:
            prev_list.append(segs[4])
    prev = _numpy_buffer(prev_list, chunk)
    buf, crcs, _ = oracle.adam_snapshot_chained(prev, params, grads, segs, chunk, hp)
    b1, b2 = np.float32(hp["beta1"]), np.float32(hp["beta2"])
    off = 0
    for k, (w_old, master, m, v) in enumerate(prev_state):
        n = master.size
        got_w = buf[off:off + 2 * n].view(np.uint16); off += 2 * n
        got_p = buf[off:off + 4 * n].view(np.float32); off += 4 * n
        got_m = buf[off:off + 4 * n].view(np.float32); off += 4 * n
        got_v = buf[off:off + 4 * n].view(np.float32); off += 4 * n
        if k == 0:
            off += segs[4].size
        assert np.array_equal(got_p, master)
        assert np.array_equal(got_m, b1 * m)
        assert np.array_equal(got_v, b2 * v)
        assert np.array_equal(got_w, _bits(torch.from_numpy(master).to(torch.bfloat16)))


def test_chained_fp16_step_counts_and_scales(oracle):
    chunk, numels = 2048, [515, 64]
    segs, params, grads, prev_state = _chained_case(13, numels, half=torch.float16)
    grads[0][5] = 0x7C00  # +inf
    grads[1][7] = 0x7E00  # NaN
    prev_list = []
    for k, grp in enumerate(prev_state):
        prev_list += list(grp)
        if k == 0:
            prev_list.append(segs[4])
    prev = _numpy_buffer(prev_list, chunk)
    inv = float(np.float32(1.0 / 512.0))
    buf, crcs, bad = oracle.adam_snapshot_chained(prev, params, grads, segs, chunk, HP, inv_scale=inv)
    assert bad == 2
    want = []
    for k, ((w, master, m, v), g) in enumerate(zip(prev_state, grads)):
        master, m, v, w = master.copy(), m.copy(), v.copy(), w.copy()
        oracle.adam_f32_f16(g, inv, master, m, v, w, **HP)
        want += [w, master, m, v]
        if k == 0:
            want.append(segs[4])
    assert np.array_equal(buf, _numpy_buffer(want, chunk))
