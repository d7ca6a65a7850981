"""Pins of the oracle's head step: brute force with explicit loops and a dense label matrix,
closed forms, finite differences of the BCE loss, slice/full consistency, brute-force top-k."""
import math

import numpy as np
import pytest
import torch

from oracle import elmo_oracle as o
from paper_2510_11168_amd import synth


def _tiny(B=6, L=40, d=8, fmt=o.BF16, seed=0, w_std=0.3):
    rng = np.random.default_rng(seed)
    X = synth.make_x(rng, B, d)
    W = o.quantize(synth.make_w0_f32(rng, L, d, w_std), fmt)
    zipf = synth.ZipfLabels(L, 1.1)
    indptr, indices = zipf.draw_csr(rng, B, "fixed5")
    return X, W, indptr, indices


def _bf16_to_float(bits):
    return torch.from_numpy(np.asarray(bits).view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()


def _e4m3_to_float(codes):
    return torch.from_numpy(np.asarray(codes)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


@pytest.mark.parametrize("fmt", [o.BF16, o.E4M3])
def test_step_against_explicit_loops(fmt):
    """Z, G, dX, dW from scalar loops over a dense Y, with decoding done by torch's casts."""
    X_bits, W_bits, indptr, indices = _tiny(fmt=fmt)
    B, d = X_bits.shape
    L = W_bits.shape[0]
    X = _bf16_to_float(X_bits)
    if fmt == o.E4M3:
        Xq = torch.from_numpy(X).to(torch.float32).to(torch.float8_e4m3fn).to(torch.float64).numpy()
        W = _e4m3_to_float(W_bits)
    else:
        Xq, W = X, _bf16_to_float(W_bits)
    Y = np.zeros((B, L))
    for i in range(B):
        for p in range(indptr[i], indptr[i + 1]):
            Y[i, indices[p]] = 1.0
    assert Y.sum() == len(indices)
    Z = np.zeros((B, L)); G = np.zeros((B, L)); dX = np.zeros((B, d)); dW = np.zeros((L, d))
    for i in range(B):
        for l in range(L):
            z = sum(Xq[i, j] * W[l, j] for j in range(d))
            Z[i, l] = z
            G[i, l] = 1.0 / (1.0 + math.exp(-z)) - Y[i, l]
    G_exact = G.copy()
    # the logit gradient is held in BF16 (Section 4.4); the independent route is torch's cast
    G = torch.from_numpy(G).to(torch.bfloat16).to(torch.float64).numpy()
    for i in range(B):
        for j in range(d):
            dX[i, j] = sum(G[i, l] * W[l, j] for l in range(L))
    for l in range(L):
        for j in range(d):
            dW[l, j] = sum(G[i, l] * X[i, j] for i in range(B))      # BF16 inputs, no 1/B
    out = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, 0, 0, fmt, 0)
    np.testing.assert_allclose(out["Z"], Z, rtol=0, atol=1e-13)
    np.testing.assert_array_equal(out["G"], G)
    exact = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, 0, 0, fmt, 0, g_exact=True)
    np.testing.assert_allclose(exact["G"], G_exact, rtol=0, atol=1e-13)
    assert 0 < np.abs(exact["G"] - out["G"]).max() <= 2.0**-9      # one BF16 rounding apart
    np.testing.assert_allclose(out["dX_partial"], dX, rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["dW"], dW, rtol=0, atol=1e-12)
    if fmt == o.E4M3:   # the two kinds of input really differ, so the test can tell them apart
        assert np.abs(Xq - X).max() > 1e-3


def test_zero_weights_closed_form():
    """W = 0: Z = 0, G = 1/2 - Y, dX = 0, dW[l] = sum_b (1/2 - y_bl) x_b, loss = B L ln 2."""
    X_bits, W_bits, indptr, indices = _tiny()
    W_bits = np.zeros_like(W_bits)
    out = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, 0, 0, o.BF16, 0)
    B, L = out["Z"].shape
    Y = o.csr_to_dense(indptr, indices, L)
    X = o.decode_bf16(X_bits)
    assert np.all(out["Z"] == 0) and np.all(out["dX_partial"] == 0)
    np.testing.assert_array_equal(out["G"], 0.5 - Y)
    np.testing.assert_allclose(out["dW"], (0.5 - Y).T @ X, atol=1e-15)
    assert abs(out["loss"] - B * L * math.log(2.0)) < 1e-9
    # and the update: w' = RNE(-lr * dW) computed in FP32
    want = o.round_bf16((-(np.float32(0.05) * out["dW"].astype(np.float32))).astype(np.float32))
    np.testing.assert_array_equal(out["W_new"], want)


def test_gradients_are_derivatives_of_the_summed_bce_loss():
    """Finite differences of the FP64 loss pin the signs, the sum (not mean) over the batch and
    the use of the old weights in dX."""
    X_bits, W_bits, indptr, indices = _tiny(B=4, L=12, d=8)
    Wd = o.decode_bf16(W_bits)
    X = o.decode_bf16(X_bits)
    Y = o.csr_to_dense(indptr, indices, 12)
    out = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, 0, 0, o.BF16, 0, g_exact=True)
    loss = lambda Xv, Wv: o.bce_loss(Xv @ Wv.T, Y)
    assert abs(loss(X, Wd) - out["loss"]) < 1e-12
    h = 1e-6
    for (i, j) in [(0, 0), (3, 7), (2, 5)]:
        Xp = X.copy(); Xp[i, j] += h
        Xm = X.copy(); Xm[i, j] -= h
        fd = (loss(Xp, Wd) - loss(Xm, Wd)) / (2 * h)
        assert abs(fd - out["dX_partial"][i, j]) < 1e-6
    for (l, j) in [(0, 0), (11, 7), (indices[0], 3)]:
        Wp = Wd.copy(); Wp[l, j] += h
        Wm = Wd.copy(); Wm[l, j] -= h
        fd = (loss(X, Wp) - loss(X, Wm)) / (2 * h)
        assert abs(fd - out["dW"][l, j]) < 1e-6


def test_bce_loss_matches_torch():
    rng = np.random.default_rng(1)
    Z = rng.standard_normal((5, 9)) * 6
    Y = (rng.random((5, 9)) < 0.2).astype(np.float64)
    ref = torch.nn.functional.binary_cross_entropy_with_logits(
        torch.from_numpy(Z), torch.from_numpy(Y), reduction="sum").item()
    assert abs(o.bce_loss(Z, Y) - ref) < 1e-10
    np.testing.assert_allclose(o.sigmoid(Z), torch.sigmoid(torch.from_numpy(Z)).numpy(), atol=1e-15)
    assert o.sigmoid(np.array([-800.0, 800.0])).tolist() == [0.0, 1.0]


@pytest.mark.parametrize("fmt,flags", [(o.BF16, 0), (o.BF16, o.FLAG_SR), (o.E4M3, o.FLAG_SR),
                                       (o.E4M3, o.FLAG_SR | o.FLAG_KAHAN), (o.BF16, o.FLAG_KAHAN)])
def test_update_rule_by_scalar_recomputation(fmt, flags):
    """The fused update re-derived element by element with Python floats forced through FP32."""
    f32 = np.float32
    X_bits, W_bits, indptr, indices = _tiny(fmt=fmt, w_std=0.05, seed=4)
    L, d = W_bits.shape
    rng = np.random.default_rng(9)
    comp = o.round_bf16((rng.standard_normal((L, d)) * 1e-3).astype(f32)) if flags & o.FLAG_KAHAN else None
    lr, seed, step = 0.05, 77, 3
    out = o.head_step(W_bits, comp, X_bits, indptr, indices, lr, seed, step, fmt, flags)
    dec = (lambda b: _bf16_to_float(b)) if fmt == o.BF16 else (lambda c: _e4m3_to_float(c))
    Wd = dec(W_bits)
    for (l, j) in [(0, 0), (1, 5), (L - 1, d - 1), (int(indices[2]), 2), (17, 4)]:
        w = f32(Wd[l, j])
        u = f32(f32(lr) * f32(out["dW"][l, j]))
        e = l * d + j
        r = None
        if flags & o.FLAG_SR:
            words = o.philox4x32_10([e // 8, 0, step, 0], [seed, 0])
            r = np.uint32((int(words[(e % 8) // 2]) >> (16 * (e % 2))) & 0xFFFF)
        if flags & o.FLAG_KAHAN:
            c = f32(_bf16_to_float(comp[l, j]))
            y = f32(f32(-u) - c)
            t = f32(w + y)
        else:
            t = f32(w - u)
        qb = o.quantize(t, fmt, r)
        assert out["W_new"][l, j] == qb
        # the stored value is one of the two grid neighbours of t
        wn = float(dec(np.array([qb]).astype(W_bits.dtype))[0])
        if fmt == o.BF16:
            assert abs(wn - float(t)) <= 2.0**-7 * abs(float(t))
        else:
            assert abs(wn - float(t)) <= max(2.0**-9, 2.0**-3 * abs(float(t)))
        if flags & o.FLAG_KAHAN:
            cn = f32(f32(f32(wn) - w) - y)
            assert out["comp_new"][l, j] == o.round_bf16(cn)
            # s - c reproduces the unrounded target to BF16 accuracy of c
            assert abs((wn - float(_bf16_to_float(out["comp_new"][l, j]))) - float(t)) <= 2.0**-8 * abs(float(cn)) + 1e-12


@pytest.mark.parametrize("fmt", [o.BF16, o.E4M3])
def test_weight_decay_is_the_l2_term_of_sgd(fmt):
    """weight_decay adds wd*w to the gradient (plain SGD with an L2 term).  Pins: (i) torch's own
    SGD step with weight_decay on FP32 copies of the same numbers, rounded to the storage format,
    gives the same codes (up to the rare element where a fused multiply-add inside torch moves the
    FP32 result across a rounding boundary); (ii) a closed form with exactly representable
    numbers; (iii) wd = 0 is the step without it, bit for bit."""
    rng = np.random.default_rng(12)
    n, d, lr, wd = 64, 32, 0.05, 0.01
    W_bits = o.quantize((rng.standard_normal((n, d)) * 0.3).astype(np.float32), fmt)
    dW = (rng.standard_normal((n, d)) * 0.5).astype(np.float32)
    elem = np.arange(n * d, dtype=np.int64).reshape(n, d)
    got, _ = o.update_rows(W_bits, None, dW, lr, fmt, 0, 0, 0, elem, weight_decay=wd)
    p = torch.nn.Parameter(torch.from_numpy(o.decode(W_bits, fmt).astype(np.float32)))
    p.grad = torch.from_numpy(dW.copy())
    torch.optim.SGD([p], lr=lr, weight_decay=wd).step()
    want = o.quantize(p.detach().numpy(), fmt)
    assert np.mean(got == want) >= 0.995
    assert np.max(np.abs(o.decode(got, fmt) - o.decode(want, fmt))) <= np.max(np.abs(o.decode(want, fmt))) * 2.0**-2
    base, _ = o.update_rows(W_bits, None, dW, lr, fmt, 0, 0, 0, elem)
    assert np.any(got != base)
    # (ii) w = 1, g = 0, lr = 1/2, wd = 1/4: t = 1 - (1/2)(0 + 1/4) = 7/8, representable in both formats
    one = o.quantize(np.ones((1, 8), np.float32), fmt)
    out, _ = o.update_rows(one, None, np.zeros((1, 8)), 0.5, fmt, 0, 0, 0, np.arange(8).reshape(1, 8), weight_decay=0.25)
    np.testing.assert_array_equal(o.decode(out, fmt), np.full((1, 8), 0.875))
    # (iii)
    zero, _ = o.update_rows(W_bits, None, dW, lr, fmt, 0, 0, 0, elem, weight_decay=0.0)
    np.testing.assert_array_equal(zero, base)


def test_classifier_dropout_is_the_gradient_of_the_masked_model():
    """Appendix "Low-Memory Dropout for Classifier".  Pins: (i) torch autograd through an explicit
    masked, rescaled copy of W (the copy the paper's kernel avoids) gives the oracle's logits, loss,
    input gradient and weight gradient -- a mask missing from one of the three products, a missing
    scale or a transposed mask fails here; (ii) threshold 0 is the step without dropout, bit for
    bit; (iii) dropped elements see a zero gradient: with RNE and no decay they do not move."""
    X_bits, W_bits, indptr, indices = _tiny(B=5, L=24, d=16)
    L, d, T, seed, step = 24, 16, 96, 5, 3
    out = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, seed, step, o.BF16, 0, g_exact=True, dropout=T)
    keep = o.dropout_keep(seed, step, np.arange(L * d).reshape(L, d), T)
    assert 0.4 < keep.mean() < 0.85
    W = torch.from_numpy(o.decode_bf16(W_bits)).requires_grad_(True)
    X = torch.from_numpy(o.decode_bf16(X_bits)).requires_grad_(True)
    Y = torch.from_numpy(o.csr_to_dense(indptr, indices, L))
    Wm = W * torch.from_numpy(keep.astype(np.float64)) * (256.0 / (256.0 - T))
    Z = X @ Wm.T
    loss = torch.nn.functional.binary_cross_entropy_with_logits(Z, Y, reduction="sum")
    loss.backward()
    np.testing.assert_allclose(out["Z"], Z.detach().numpy(), rtol=0, atol=1e-12)
    assert abs(out["loss"] - loss.item()) < 1e-10
    np.testing.assert_allclose(out["dX_partial"], X.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(out["dW"], W.grad.numpy(), rtol=0, atol=1e-12)
    assert np.all(out["dW"][~keep] == 0.0) and np.any(out["dW"][keep] != 0.0)
    # (ii)
    a = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, seed, step, o.BF16, o.FLAG_SR)
    b = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, seed, step, o.BF16, o.FLAG_SR, dropout=0)
    np.testing.assert_array_equal(a["W_new"], b["W_new"])
    np.testing.assert_array_equal(a["dX_partial"], b["dX_partial"])
    # (iii)
    c = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, seed, step, o.BF16, 0, dropout=T)
    np.testing.assert_array_equal(c["W_new"][~keep], W_bits[~keep])
    assert np.any(c["W_new"][keep] != W_bits[keep])


def test_dropout_mask_stream():
    """The keep mask: (i) byte b of a block is byte b of the generator's four little-endian output
    words, checked through a byte view of the words; (ii) the drop rate is threshold/256 (a
    binomial bound over 2^20 elements), for every block position alike; (iii) masks of different
    steps and seeds differ, the same (seed, step) repeats, and a subset of elements gives the same
    bits as the full range; (iv) the mask blocks are not the blocks of the rounding fields."""
    seed, step = 0x1234567890ABCDEF, 77
    elem = np.arange(64, dtype=np.int64)
    ctr = np.array([[b, 0, step, 0x80000000] for b in range(4)], dtype=np.uint64)
    key = np.array([seed & 0xFFFFFFFF, seed >> 32], dtype=np.uint64)
    raw = np.ascontiguousarray(o.philox4x32_10(ctr, key).astype("<u4")).view(np.uint8).reshape(-1)
    for T in (1, 64, 200, 255):
        np.testing.assert_array_equal(o.dropout_keep(seed, step, elem, T), raw >= T)
    assert o.dropout_keep(seed, step, elem, 0).all()
    n = 1 << 20
    big = np.arange(n, dtype=np.int64)
    for T in (26, 128, 230):
        keep = o.dropout_keep(seed, step, big, T)
        p = T / 256
        assert abs((~keep).mean() - p) < 5 * math.sqrt(p * (1 - p) / n)
        per_pos = (~keep).reshape(-1, 16).mean(axis=0)
        assert np.all(np.abs(per_pos - p) < 5 * math.sqrt(p * (1 - p) / (n / 16)))
    k0 = o.dropout_keep(seed, step, big[:4096], 128)
    assert 0.4 < np.mean(k0 != o.dropout_keep(seed, step + 1, big[:4096], 128)) < 0.6
    assert 0.4 < np.mean(k0 != o.dropout_keep(seed + 1, step, big[:4096], 128)) < 0.6
    np.testing.assert_array_equal(k0, o.dropout_keep(seed, step, big[:4096], 128))
    sub = np.array([4095, 17, 16, 15, 1000], dtype=np.int64)
    np.testing.assert_array_equal(o.dropout_keep(seed, step, sub, 128), k0[sub])
    # (iv) block 0 of the rounding fields at the same (seed, step) is another Philox output
    sr_words = o.philox4x32_10(np.array([0, 0, step, 0], dtype=np.uint64), key)
    assert not np.array_equal(np.ascontiguousarray(sr_words.astype("<u4")).view(np.uint8), raw[:16])
    with pytest.raises(ValueError):
        o.dropout_keep(seed, 1 << 63, elem, 10)
    with pytest.raises(ValueError):
        o.dropout_keep(seed, step, elem, 256)


def test_rne_cancels_small_updates_bit_identically():
    """Section 4.1: with round-to-nearest and a tiny learning rate the weights do not move."""
    X_bits, W_bits, indptr, indices = _tiny(w_std=0.3)
    out = o.head_step(W_bits, None, X_bits, indptr, indices, 1e-6, 0, 0, o.BF16, 0)
    moved = out["W_new"] != W_bits
    small = np.abs(o.decode_bf16(W_bits)) > 1e-2
    assert not np.any(moved & small)
    # with SR the same step moves some weights, and the mean over seeds follows the FP32 target
    outs = [o.decode_bf16(o.head_step(W_bits, None, X_bits, indptr, indices, 1e-3, s, 0, o.BF16,
                                      o.FLAG_SR)["W_new"]) for s in range(400)]
    mean = np.mean(outs, axis=0)
    target = o.decode_bf16(W_bits) - 1e-3 * out["dW"]
    gap = 2.0**-7 * np.abs(o.decode_bf16(W_bits)) + 1e-30
    assert np.max(np.abs(mean - target) / gap) < 0.15   # ~4.5 sigma of 0.5/sqrt(400)
    assert np.any(outs[0] != o.decode_bf16(W_bits))


def test_label_subset_gives_rows_of_full_result():
    """Rows of W evaluated alone (with their global ids) equal the same rows of the full step --
    the property that makes label chunking exact and lets large heads be checked by sampling."""
    fmt, flags = o.E4M3, o.FLAG_SR | o.FLAG_KAHAN
    X_bits, W_bits, indptr, indices = _tiny(L=64, fmt=fmt, w_std=0.05)
    comp = np.zeros(W_bits.shape, np.uint16)
    full = o.head_step(W_bits, comp, X_bits, indptr, indices, 0.05, 5, 9, fmt, flags)
    ids = np.array([0, 3, 17, int(indices[0]), 63])
    ids = np.unique(ids)
    part = o.head_step(W_bits[ids], comp[ids], X_bits, indptr, indices, 0.05, 5, 9, fmt, flags,
                       label_ids=ids)
    np.testing.assert_array_equal(part["W_new"], full["W_new"][ids])
    np.testing.assert_array_equal(part["comp_new"], full["comp_new"][ids])
    np.testing.assert_array_equal(part["G"], full["G"][:, ids])
    # chunked accumulation of dX equals the full dX
    acc = np.zeros_like(full["dX_partial"])
    for c0 in range(0, 64, 24):
        cid = np.arange(c0, min(64, c0 + 24))
        acc += o.head_step(W_bits[cid], comp[cid], X_bits, indptr, indices, 0.05, 5, 9, fmt, flags,
                           label_ids=cid)["dX_partial"]
    np.testing.assert_allclose(acc, full["dX_partial"], atol=1e-12)
    dX_rows, Z_rows = o.input_gradient_rows(W_bits, X_bits, indptr, indices, fmt, [1, 4], block=24)
    np.testing.assert_allclose(dX_rows, full["dX_partial"][[1, 4]], atol=1e-12)
    np.testing.assert_allclose(Z_rows, full["Z"][[1, 4]], atol=1e-13)


@pytest.mark.parametrize("fmt", [o.BF16, o.E4M3])
def test_head_only_kahan_is_kahan_on_the_prefix_and_plain_elsewhere(fmt):
    """Kahan summation for head labels (appendix "Precision Recovery for Sensitive Applications"):
    a label's update depends on no other label, so with compensation on labels < k only, those rows
    must equal the rows of the all-Kahan step and the others the rows of the step without
    compensation; k = L and k = 0 are the two plain modes themselves."""
    L, k = 64, 24
    X_bits, W_bits, indptr, indices = _tiny(L=L, fmt=fmt, w_std=0.05)
    rng = np.random.default_rng(3)
    comp = o.round_bf16((rng.standard_normal(W_bits.shape) * 1e-4).astype(np.float32))
    flags = o.FLAG_SR | o.FLAG_KAHAN
    args = (X_bits, indptr, indices, 0.05, 7, 2, fmt)
    allk = o.head_step(W_bits, comp, *args, flags)
    none = o.head_step(W_bits, None, *args, o.FLAG_SR)
    head = o.head_step(W_bits, comp, *args, flags, kahan_rows=k)
    np.testing.assert_array_equal(head["W_new"][:k], allk["W_new"][:k])
    np.testing.assert_array_equal(head["comp_new"][:k], allk["comp_new"][:k])
    np.testing.assert_array_equal(head["W_new"][k:], none["W_new"][k:])
    np.testing.assert_array_equal(head["comp_new"][k:], comp[k:])          # untouched
    assert np.any(allk["W_new"][k:] != none["W_new"][k:])                  # the two modes do differ
    np.testing.assert_array_equal(head["dX_partial"], allk["dX_partial"])  # gradients do not depend on it
    full = o.head_step(W_bits, comp, *args, flags, kahan_rows=L)
    np.testing.assert_array_equal(full["W_new"], allk["W_new"])
    np.testing.assert_array_equal(full["comp_new"], allk["comp_new"])
    zero = o.head_step(W_bits, comp, *args, flags, kahan_rows=0)
    np.testing.assert_array_equal(zero["W_new"], none["W_new"])
    # a label subset straddling the boundary still gives the rows of the full result
    ids = np.array([3, 23, 24, 40])
    part = o.head_step(W_bits[ids], comp[ids], *args, flags, label_ids=ids, kahan_rows=k)
    np.testing.assert_array_equal(part["W_new"], head["W_new"][ids])
    np.testing.assert_array_equal(part["comp_new"], head["comp_new"][ids])


def test_different_steps_draw_different_roundings_same_step_repeats():
    X_bits, W_bits, indptr, indices = _tiny(fmt=o.E4M3, w_std=0.05)
    a = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, 1, 0, o.E4M3, o.FLAG_SR)["W_new"]
    b = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, 1, 0, o.E4M3, o.FLAG_SR)["W_new"]
    c = o.head_step(W_bits, None, X_bits, indptr, indices, 0.05, 1, 1, o.E4M3, o.FLAG_SR)["W_new"]
    assert np.array_equal(a, b) and not np.array_equal(a, c)


def test_topk_brute_force():
    rng = np.random.default_rng(2)
    Z = rng.standard_normal((7, 300)).round(1)      # rounding creates ties
    idx, val = o.topk(Z, 10)
    for i in range(7):
        order = sorted(range(300), key=lambda l: (-Z[i, l], l))[:10]
        assert idx[i].tolist() == order
        assert val[i].tolist() == [Z[i, l] for l in order]


def test_precision_hits_on_a_worked_example():
    """P@k = (1/k) sum_{l in top_k} y_l (evaluation section).  Two rows, k = 3, counted by hand:
    row 0 truth {2, 5}, predictions (5, 1, 2) -> hits after 1, 2, 3 predictions: 1, 1, 2;
    row 1 truth {0},    predictions (3, 0, 4) -> 0, 1, 1."""
    indptr, indices = np.array([0, 2, 3]), np.array([2, 5, 0])
    idx = np.array([[5, 1, 2], [3, 0, 4]])
    hits = o.precision_hits(idx, indptr, indices)
    np.testing.assert_array_equal(hits, [1, 2, 3])
    p_at = hits / (np.arange(1, 4) * 2)
    np.testing.assert_allclose(p_at, [0.5, 0.5, 0.5])
    # perfect predictions: every true label first -> P@k = min(k, n_i) / k averaged over the rows
    idx = np.array([[2, 5, 9], [0, 7, 8]])
    np.testing.assert_array_equal(o.precision_hits(idx, indptr, indices), [2, 3, 3])
    # scores that rank the positives first give P@1 = 1 through the oracle's own top-k
    Z = np.full((2, 10), -1.0)
    Z[0, [2, 5]] = [3.0, 2.0]
    Z[1, 0] = 1.0
    top, _ = o.topk(Z, 3)
    assert o.precision_hits(top, indptr, indices)[0] == 2


def test_synthetic_label_recipe():
    zipf = synth.ZipfLabels(1000, 1.0)
    rng = np.random.default_rng(0)
    indptr, indices = zipf.draw_csr(rng, 500, "poisson4.5")
    assert indptr[0] == 0 and indptr[-1] == len(indices) and indices.dtype == np.int32
    for i in range(500):
        row = indices[indptr[i]:indptr[i + 1]]
        assert len(row) >= 1 and np.all(np.diff(row) > 0) and row.min() >= 0 and row.max() < 1000
    counts = np.bincount(indices, minlength=1000)
    assert counts[:10].sum() > counts[500:510].sum() * 5        # long-tailed: head labels dominate
    X = synth.make_x(rng, 4, 768)
    assert np.allclose(np.linalg.norm(o.decode_bf16(X), axis=1), 1.0, atol=5e-3)
