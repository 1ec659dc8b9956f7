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
