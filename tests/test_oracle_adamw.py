"""Pins of the oracle's Kahan-AdamW (Section 4.1: Kahan summation for the encoder's parameters)
against things other than itself: torch's AdamW, the exact arithmetic it approximates, and the
property the compensation exists for."""
import numpy as np
import torch

from oracle import elmo_oracle as o


def _bits(x):
    return o.round_bf16(np.asarray(x, dtype=np.float32))


def test_wide_recipe_is_torch_adamw():
    """The FP64, nothing-rounded form of the recipe against torch.optim.AdamW in float64 over five
    steps: decoupled decay, both bias corrections, eps outside the square root."""
    rng = np.random.default_rng(0)
    n, lr, b1, b2, eps, wd = 500, 1e-2, 0.9, 0.98, 1e-6, 0.05
    p = rng.standard_normal(n) * 0.1
    P = torch.nn.Parameter(torch.from_numpy(p.copy()))
    opt = torch.optim.AdamW([P], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    c, m, v = np.zeros(n), np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        g = rng.standard_normal(n) * np.exp(rng.uniform(-3, 1, n))
        P.grad = torch.from_numpy(g.copy())
        opt.step()
        p, c, m, v = o.kahan_adamw(p, c, m, v, g, lr, b1, b2, eps, wd, t, wide=True)
        np.testing.assert_allclose(p, P.detach().numpy(), rtol=0, atol=1e-14)
        st = opt.state[P]
        np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=0, atol=1e-15)
        np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=0, atol=1e-15)


def test_rounded_recipe_follows_the_wide_one():
    """One step from BF16 inputs: the stored parameter is the BF16 neighbour of the exact result,
    the pair (p', c') represents it to about BF16-squared accuracy, and BF16 moments are the
    round-to-nearest of the FP32 ones."""
    rng = np.random.default_rng(1)
    n, lr, b1, b2, eps, wd, t = 4000, 3e-3, 0.9, 0.999, 1e-8, 0.01, 7
    pb, gb = _bits(rng.standard_normal(n) * 0.2), _bits(rng.standard_normal(n) * 0.05)
    m32 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    v32 = (rng.random(n) * 1e-3).astype(np.float32)
    cb = np.zeros(n, np.uint16)
    pn, cn, m1, v1 = o.kahan_adamw(pb, cb, m32, v32, gb, lr, b1, b2, eps, wd, t)
    wp, _, wm, wv = o.kahan_adamw(o.decode_bf16(pb), np.zeros(n), m32.astype(np.float64), v32.astype(np.float64),
                                  o.decode_bf16(gb), lr, b1, b2, eps, wd, t, wide=True)
    assert m1.dtype == np.float32 and v1.dtype == np.float32
    np.testing.assert_allclose(m1, wm, rtol=3e-7, atol=1e-8)
    np.testing.assert_allclose(v1, wv, rtol=3e-7)
    assert np.mean(pn == _bits(wp)) > 0.99                      # FP32 rounding of s may flip a tie now and then
    np.testing.assert_allclose(o.decode_bf16(pn), wp, rtol=2.0**-8)
    held = o.decode_bf16(pn) - o.decode_bf16(cn)               # what the pair stands for
    assert np.max(np.abs(held - wp) / np.abs(wp)) < 2.0**-14
    # BF16 moments: same arithmetic, stored rounded
    mb, vb = _bits(m32), _bits(v32)
    pn2, cn2, m2, v2 = o.kahan_adamw(pb, cb, mb, vb, gb, lr, b1, b2, eps, wd, t)
    assert m2.dtype == np.uint16 and v2.dtype == np.uint16
    _, _, m2f, v2f = o.kahan_adamw(pb, cb, o.decode_bf16(mb).astype(np.float32), o.decode_bf16(vb).astype(np.float32), gb,
                                   lr, b1, b2, eps, wd, t)
    np.testing.assert_array_equal(m2, _bits(m2f))
    np.testing.assert_array_equal(v2, _bits(v2f))


def test_first_step_moves_by_the_learning_rate():
    """t = 1, no decay, eps = 0: the bias-corrected ratio is g / |g|, so every parameter moves by
    lr against the sign of its gradient (to BF16 accuracy)."""
    g = np.array([1.0, -2.0, 0.5, -0.125], np.float32)
    p = np.array([1.0, 1.0, -3.0, 0.75], np.float32)
    z = np.zeros(4, np.float32)
    pn, cn, _, _ = o.kahan_adamw(_bits(p), np.zeros(4, np.uint16), z, z, _bits(g), 0.25, 0.9, 0.999, 0.0, 0.0, 1)
    want = p - 0.25 * np.sign(g)
    assert np.max(np.abs(o.decode_bf16(pn) - o.decode_bf16(cn) - want)) < 2.0**-20
    np.testing.assert_allclose(o.decode_bf16(pn), want, rtol=2.0**-8)


def test_compensation_keeps_updates_that_bf16_alone_cancels():
    """Section 4.1: with BF16 parameters and round-to-nearest, steps below half a grid spacing are
    lost.  400 steps of lr = 1e-4 on parameters near 1 (spacing 2^-7, so every step is 1/39 of
    half a spacing): without compensation the parameters never move; with it they follow torch's
    FP32 AdamW through five spacings of drift to within one spacing, and p - c follows it to within
    2.5 % of the drift (each step rounds the BF16 compensation, about 1e-5 here, a random walk)."""
    rng = np.random.default_rng(2)
    n, lr, b1, b2, eps = 256, 1e-4, 0.9, 0.999, 1e-8
    p0 = (1.0 + rng.random(n) * 0.5).astype(np.float32)
    pb = _bits(p0)
    P = torch.nn.Parameter(torch.from_numpy(o.decode_bf16(pb).astype(np.float32)))
    opt = torch.optim.AdamW([P], lr=lr, betas=(b1, b2), eps=eps, weight_decay=0.0)
    pk, ck = pb.copy(), np.zeros(n, np.uint16)
    pl = pb.copy()
    mk = np.zeros(n, np.float32); vk = np.zeros(n, np.float32)
    ml = np.zeros(n, np.float32); vl = np.zeros(n, np.float32)
    for t in range(1, 401):
        g = (1.0 + 0.1 * rng.standard_normal(n)).astype(np.float32)      # steady drift downwards
        gb = _bits(g)
        P.grad = torch.from_numpy(o.decode_bf16(gb).astype(np.float32))
        opt.step()
        pk, ck, mk, vk = o.kahan_adamw(pk, ck, mk, vk, gb, lr, b1, b2, eps, 0.0, t)
        pl, _, ml, vl = o.kahan_adamw(pl, np.zeros(n, np.uint16), ml, vl, gb, lr, b1, b2, eps, 0.0, t)
    ref = P.detach().numpy().astype(np.float64)
    drift = o.decode_bf16(pb) - ref
    assert np.all(drift > 3.5e-2)                                         # about 400 * 1e-4
    np.testing.assert_array_equal(pl, pb)                                 # plain BF16: every step cancelled
    assert np.max(np.abs(o.decode_bf16(pk) - ref)) <= 2.0**-7            # Kahan: within one spacing
    assert np.max(np.abs(o.decode_bf16(pk) - o.decode_bf16(ck) - ref)) < 1e-3
