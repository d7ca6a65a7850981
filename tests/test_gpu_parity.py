"""GPU parity: the HIP path (called through the C ABI) against the CPU oracle on the same seeded
inputs.  Bars (from the benchmark spec):
  * quantisation / stochastic-rounding kernels: bit-exact on identical FP32 inputs;
  * logits-derived quantities and dX: relative Frobenius error <= 2e-2 (BF16) / 6e-2 (FP8);
  * updated weights: within 1 unit in the last place of the storage format for >= 99.9 % of the
    elements after one step (same random fields on both sides).
"""
import sys

import numpy as np
import pytest
import torch

from oracle import elmo_oracle as o
from paper_2510_11168_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def b():
    from paper_2510_11168_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to(DEV)


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def ordered(bits, fmt):
    """Monotone integer index of a sign-magnitude code: neighbours on the grid differ by 1."""
    bits = np.asarray(bits).astype(np.int64)
    if fmt == o.BF16:
        mag, neg = bits & 0x7FFF, (bits >> 15) & 1
    else:
        mag, neg = bits & 0x7F, (bits >> 7) & 1
    return np.where(neg == 1, -mag, mag)


def assert_far_misses_are_tiny(Wn, Wref, dist, fmt, lr):
    """Beyond the 1-ulp bar: where the two sides differ by more than two grid steps the weight
    must sit next to zero, where a grid step is far smaller than the update itself.  There the
    difference is bounded in absolute terms: one BF16 step of one logit-gradient term times |x|
    (|x| < 1 after L2 normalisation), times lr."""
    far = dist > 2
    if np.any(far):
        diff = np.abs(o.decode(Wn, fmt) - o.decode(Wref, fmt))[far]
        assert diff.max() <= lr * 2.0**-8, f"largest far miss {diff.max():.3e}"


def rel_fro(a, ref):
    return float(np.linalg.norm(np.asarray(a, np.float64) - ref) / max(np.linalg.norm(ref), 1e-300))


# dX: the contract is a relative Frobenius error of 2e-2 (BF16) / 6e-2 (FP8) over the whole matrix.
# One completely wrong sample row of a 1024-row batch moves that norm by only 1/32, so the bound is
# also taken row by row, and both are held to what the arithmetic gives when the two sides start
# from the same bits: G and dX_out are rounded to BF16 (unit roundoff 2^-9), measured 1.7e-3.
DX_SHARP, DX_SHARP_ROW = 6e-3, 1e-2


def row_errors(a, ref):
    a, ref = np.atleast_2d(np.asarray(a, np.float64)), np.atleast_2d(ref)
    num, den = np.linalg.norm(a - ref, axis=1), np.linalg.norm(ref, axis=1)
    return np.where(den > 0, num / np.where(den > 0, den, 1.0), np.where(num > 0, np.inf, 0.0))


def assert_dx_close(dX, ref, tol, what="dX"):
    """Whole-matrix contract bound, the same-operand bound, and the same-operand bound per row."""
    e, rows = rel_fro(dX, ref), row_errors(dX, ref)
    say(f"   {what}: rel-Fro {e:.2e}; worst row {rows.max():.2e} (row {int(rows.argmax())} of {len(rows)})")
    assert e <= tol and e <= DX_SHARP, f"{what}: relative Frobenius error {e:.3e}"
    assert rows.max() <= DX_SHARP_ROW, f"{what}: row {int(rows.argmax())} is off by {rows.max():.3e}"
    return e


# --------------------------------------------------------------------------------- quantisers
def _quant_inputs():
    rng = np.random.default_rng(11)
    n = 1 << 21
    x = (rng.standard_normal(n) * np.exp(rng.uniform(-20, 8, n))).astype(np.float32)
    # every FP32 exponent with random mantissas, exact grid points, ties, zeros, overflow, inf, NaN
    exps = np.repeat(np.arange(0, 255, dtype=np.uint32), 64)
    man = rng.integers(0, 1 << 23, size=exps.size, dtype=np.uint32)
    sign = rng.integers(0, 2, size=exps.size, dtype=np.uint32)
    allexp = ((sign << 31) | (exps << 23) | man).view(np.float32)
    grid = o.decode_e4m3(np.arange(256, dtype=np.uint8))
    grid = grid[~np.isnan(grid)].astype(np.float32)
    ties = ((grid[:-1].astype(np.float64) + grid[1:].astype(np.float64)) / 2).astype(np.float32)
    special = np.array([0.0, -0.0, 448.0, 464.0, 465.0, 1e9, -1e9, np.inf, -np.inf, np.nan, 3.4e38, -3.4e38,
                        1e-45, -1e-45, 2.0**-10, 3 * 2.0**-10, 2.0**-6, 2.0**-6 - 2.0**-20], dtype=np.float32)
    return np.concatenate([x, allexp, grid, ties, special])


@pytest.mark.parametrize("fmt", [o.BF16, o.E4M3])
@pytest.mark.parametrize("mode", [0, 1])
def test_quantize_bit_exact(b, fmt, mode):
    x = _quant_inputs()
    n = x.size
    seed, step, first = 0x1234567890ABCDEF, 0xFEDCBA9876543210, (1 << 40) + 5      # odd offset: all fields
    say(f"[quantize] fmt={fmt} mode={mode} n={n}")
    src = torch.from_numpy(x).to(DEV)
    dst = torch.zeros(n, dtype=torch.int16 if fmt == o.BF16 else torch.uint8, device=DEV)
    b.elmo_quantize(src, n, fmt, mode, seed, step, first, dst)
    torch.cuda.synchronize()
    got = dst.cpu().numpy()
    got = got.view(np.uint16) if fmt == o.BF16 else got
    r = o.sr_fields(seed, step, first + np.arange(n, dtype=np.uint64)) if mode else None
    want = o.quantize(x, fmt, r)
    bad = np.nonzero(got != want)[0]
    assert bad.size == 0, f"{bad.size} mismatches, first at {bad[0]}: x={x[bad[0]]!r} got={got[bad[0]]:#x} want={want[bad[0]]:#x}"


@pytest.mark.parametrize("E,M", [(8, 7), (5, 10), (5, 2), (4, 3), (3, 4), (2, 1), (6, 9), (8, 22)])
@pytest.mark.parametrize("mode", [0, 1])
def test_simulated_format_quantiser_bit_exact(b, E, M, mode):
    """The (exponent, mantissa) format simulator against the oracle on the same 2.1 M inputs as the
    storage-format quantisers (every FP32 exponent, ties, +-0, subnormals, overflow, inf, NaN)."""
    x = _quant_inputs()
    n = x.size
    seed, step, first = 0x0F1E2D3C4B5A6978, 3, (1 << 33) + 3
    say(f"[quantize E{E}M{M}] mode={mode} n={n}")
    src = torch.from_numpy(x).to(DEV)
    dst = torch.zeros(n, dtype=torch.float32, device=DEV)
    b.elmo_quantize_em(src, n, E, M, mode, seed, step, first, dst)
    torch.cuda.synchronize()
    got = dst.cpu().numpy()
    r = o.sr_fields(seed, step, first + np.arange(n, dtype=np.uint64)) if mode else None
    want = o.round_em(x, E, M, r)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    bad = np.nonzero((got.view(np.uint32) != want.view(np.uint32)) & ~nan)[0]
    assert bad.size == 0, f"{bad.size} mismatches, first at {bad[0]}: x={x[bad[0]]!r} got={got[bad[0]]!r} want={want[bad[0]]!r}"


def test_quantize_empty_is_a_no_op(b):
    b.elmo_quantize(None, 0, o.BF16, 0, 0, 0, 0, None)


@pytest.mark.parametrize("state_bf16", [True, False])
@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_kahan_adamw_bit_exact(b, state_bf16, wd):
    """Three consecutive AdamW steps with Kahan-compensated BF16 parameters on 1 M + 5 elements
    (the vector body and the scalar tail), values over many binades, BF16 and FP32 moments:
    parameters, compensation and moments bit for bit against the oracle after every step."""
    rng = np.random.default_rng(13)
    n = (1 << 20) + 5
    lr, b1, b2, eps = 2e-3, 0.9, 0.999, 1e-8
    pb = o.round_bf16((rng.standard_normal(n) * np.exp(rng.uniform(-6, 2, n))).astype(np.float32))
    cb = np.zeros(n, np.uint16)
    m = np.zeros(n, np.uint16 if state_bf16 else np.float32)
    v = np.zeros(n, np.uint16 if state_bf16 else np.float32)
    P, C = dev(pb), dev(cb)
    M, V = dev(m), dev(v)
    sd = b.ELMO_BF16 if state_bf16 else b.ELMO_FP32
    say(f"[kahan-adamw] state_bf16={state_bf16} wd={wd} n={n}")
    for t in range(1, 4):
        gb = o.round_bf16((rng.standard_normal(n) * np.exp(rng.uniform(-8, 1, n))).astype(np.float32))
        if t == 2:
            gb[:1000] = 0                      # zero gradients: the moments decay, sqrt(v) + eps stays positive
        b.elmo_kahan_adamw(P, C, M, V, dev(gb), n, sd, lr, b1, b2, eps, wd, t)
        torch.cuda.synchronize()
        pb, cb, m, v = o.kahan_adamw(pb, cb, m, v, gb, lr, b1, b2, eps, wd, t)
        got_m = host_u16(M) if state_bf16 else M.cpu().numpy()
        got_v = host_u16(V) if state_bf16 else V.cpu().numpy()
        for name, got, want in (("p", host_u16(P), pb), ("c", host_u16(C), cb), ("m", got_m, m), ("v", got_v, v)):
            w32 = want.view(np.uint32) if want.dtype == np.float32 else want
            g32 = got.view(np.uint32) if got.dtype == np.float32 else got
            bad = np.nonzero(g32 != w32)[0]
            assert bad.size == 0, f"step {t} {name}: {bad.size} mismatches, first at {bad[0]}: got {got[bad[0]]!r} want {want[bad[0]]!r}"
    b.elmo_kahan_adamw(None, None, None, None, None, 0, sd, lr, b1, b2, eps, wd, 1)      # n = 0 is a no-op


# --------------------------------------------------------------------------------- head step
class Case:
    """A head on the device initialised from host bits, plus the host copies the oracle needs."""

    def __init__(self, b, L, d, fmt, chunk, flags, B, max_nnz=None, seed=0, w_std=0.02, comp_std=0.0, kahan_rows=0,
                 weight_decay=0.0, dropout_p=0.0):
        rng = np.random.default_rng([seed, L, d])
        self.b, self.L, self.d, self.fmt, self.flags = b, L, d, fmt, flags
        self.W0 = o.quantize(synth.make_w0_f32(rng, L, d, w_std), fmt)
        self.C0 = None
        if flags & o.FLAG_KAHAN:
            self.C0 = o.round_bf16((rng.standard_normal((kahan_rows or L, d)) * comp_std).astype(np.float32))
        self.head = b.Head(L, d, fmt, chunk, flags, B, max_nnz or 64 * B, kahan_rows=kahan_rows, weight_decay=weight_decay,
                           dropout_p=dropout_p)
        self.load(self.W0, self.C0)

    def load(self, W, C):
        self.head.weights().copy_(dev(W))
        if C is not None:
            self.head.compensation().copy_(dev(C))

    def W(self):
        w = self.head.weights().cpu().numpy()
        return w.view(np.uint16) if self.fmt == o.BF16 else w

    def C(self):
        return None if self.head.comp is None else host_u16(self.head.compensation())

    def step(self, X, indptr, indices, lr, seed, step, want_dx=True, want_loss=True):
        Xd, ip, ix = dev(X), dev(indptr), dev(indices)
        dX = torch.zeros(X.shape, dtype=torch.int16, device=DEV) if want_dx else None
        loss = torch.zeros(1, dtype=torch.float32, device=DEV) if want_loss else None
        self.head.step(Xd, ip, ix, lr, seed, step, dX, loss)
        torch.cuda.synchronize()
        return (None if dX is None else o.decode_bf16(host_u16(dX)),
                None if loss is None else float(loss.item()))


def check_step(case, X, indptr, indices, lr, seed, step, tol, W_before=None, C_before=None, want_loss=True):
    """Run one GPU step and compare everything with the oracle fed the same starting bits."""
    W_before = case.W() if W_before is None else W_before
    C_before = case.C() if C_before is None else C_before
    dX, loss = case.step(X, indptr, indices, lr, seed, step, want_loss=want_loss)
    ref = o.head_step(W_before, C_before, X, indptr, indices, lr, seed, step, case.fmt, case.flags)
    Wn = case.W()
    dist = np.abs(ordered(Wn, case.fmt) - ordered(ref["W_new"], case.fmt))
    frac_exact = float(np.mean(dist == 0))
    frac_1ulp = float(np.mean(dist <= 1))
    e_loss = abs(loss - ref["loss"]) / abs(ref["loss"]) if want_loss else 0.0
    say(f"   W': exact {frac_exact:.5f}, within 1 ulp {frac_1ulp:.6f}, max {dist.max()};  loss rel {e_loss:.2e}")
    assert frac_1ulp >= 0.999
    assert_far_misses_are_tiny(Wn, ref["W_new"], dist, case.fmt, lr)
    assert_dx_close(dX, ref["dX_partial"], tol)
    assert e_loss <= 2e-3
    if case.flags & o.FLAG_KAHAN:
        # compensation: compare the value the pair (w', c') represents, w' - c', with the oracle's
        same = dist == 0
        cg, cr = o.decode_bf16(case.C()), o.decode_bf16(ref["comp_new"])
        scale = np.maximum(np.abs(o.decode(ref["W_new"], case.fmt)), 2.0**-9)
        err = np.abs(cg - cr)[same] / scale[same]
        say(f"   comp: max |c - c_ref| / |w| on identical w' = {err.max():.2e}")
        assert np.quantile(err, 0.999) <= 2.0**-8
    return ref


def test_tiny_config_three_steps(b):
    """Benchmark configuration 1: L=8192, d=256, B=64, BF16 + SR, chunk 2048, lr 0.05, 3 steps."""
    cfg = synth.CONFIGS["tiny"]
    case = Case(b, cfg.L, cfg.d, cfg.fmt, cfg.chunk, cfg.flags, cfg.B)
    zipf = synth.ZipfLabels(cfg.L, cfg.zipf_s)
    for step in range(cfg.steps):
        X, indptr, indices = synth.make_batch(cfg, step, zipf)
        say(f"[tiny] step {step} nnz={len(indices)}")
        check_step(case, X, indptr, indices, cfg.lr, 0, step, 2e-2)


@pytest.mark.parametrize("fmt,flags,tol", [
    (o.E4M3, o.FLAG_SR | o.FLAG_KAHAN, 6e-2),
    (o.E4M3, o.FLAG_SR, 6e-2),
    (o.E4M3, 0, 6e-2),
    (o.BF16, o.FLAG_KAHAN, 2e-2),
    (o.BF16, 0, 2e-2),
])
def test_ragged_shapes_all_modes(b, fmt, flags, tol):
    """Labels and batch that are no multiple of any tile, several chunks with a short last one,
    non-zero compensation on entry."""
    L, d, B, chunk = 5 * 128 + 77, 256, 70, 256
    case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.05, comp_std=2e-4, seed=3)
    rng = np.random.default_rng(5)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    say(f"[ragged] fmt={fmt} flags={flags} L={L} B={B} chunk={chunk} nnz={len(indices)}")
    check_step(case, X, indptr, indices, 0.1, 42, 7, tol)


@pytest.mark.parametrize("fmt,flags,d,tol", [
    (o.E4M3, o.FLAG_SR | o.FLAG_KAHAN, 384, 6e-2),
    (o.E4M3, o.FLAG_SR, 256, 6e-2),
    (o.BF16, o.FLAG_KAHAN, 384, 2e-2),
    (o.BF16, o.FLAG_SR, 128, 2e-2),
])
def test_large_batch_kernels_on_ragged_tiles(b, fmt, flags, d, tol):
    """Batches above 128 rows take the three separate 256 x 256-tile kernels.  Element-by-element
    parity where nothing is a multiple of a tile: 300 samples (two batch tiles, the second one
    mostly padding), widths with a half column tile (384, 128), three label tiles with a ragged
    tail, two chunks of different length, non-zero compensation on entry."""
    L, B, chunk = 3 * 256 + 77, 300, 512
    case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.05, comp_std=2e-4, seed=6)
    rng = np.random.default_rng(11)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    say(f"[large-batch ragged] fmt={fmt} flags={flags} L={L} d={d} B={B} chunk={chunk} nnz={len(indices)}")
    check_step(case, X, indptr, indices, 0.1, 17, 3, tol)


@pytest.mark.parametrize("d,B", [(1024, 300), (1024, 70), (640, 70), (1536, 130)])
def test_wider_embeddings(b, d, B):
    """Embedding widths with four and six 256-column tiles and one that is no multiple of 256
    (640: the small batch then takes the separate kernels), in both batch regimes."""
    L, chunk = 2 * 256 + 77, 384
    fmt, flags = o.E4M3, o.FLAG_SR | o.FLAG_KAHAN
    case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.05, comp_std=2e-4, seed=41)
    rng = np.random.default_rng(43)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    say(f"[wide] d={d} B={B} L={L} chunk={chunk}")
    check_step(case, X, indptr, indices, 0.1, 3, 2, 6e-2)


@pytest.mark.parametrize("B", [70, 300])
def test_kahan_for_head_labels_only(b, B):
    """Compensation on the first 256 labels only, boundary inside the second chunk (384 labels per
    chunk), for the single-pass small-batch kernel (B = 70) and the separate kernels (B = 300):
    head rows against the oracle's Kahan update with their compensation, the other rows against
    its plain update."""
    L, d, chunk, k = 5 * 128 + 77, 256, 384, 256
    fmt, flags = o.E4M3, o.FLAG_SR | o.FLAG_KAHAN
    case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.05, comp_std=2e-4, seed=9, kahan_rows=k)
    assert case.head.compensation().shape == (k, d)
    rng = np.random.default_rng(21)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    say(f"[head-only kahan] B={B} L={L} kahan_rows={k} chunk={chunk}")
    C_pad = np.zeros((L, d), np.uint16)
    C_pad[:k] = case.C0
    dX, loss = case.step(X, indptr, indices, 0.1, 3, 5)
    ref = o.head_step(case.W0, C_pad, X, indptr, indices, 0.1, 3, 5, fmt, flags, kahan_rows=k)
    Wn = case.W()
    dist = np.abs(ordered(Wn, fmt) - ordered(ref["W_new"], fmt))
    say(f"   W': within 1 ulp head {np.mean(dist[:k] <= 1):.6f}, rest {np.mean(dist[k:] <= 1):.6f}")
    assert np.mean(dist[:k] <= 1) >= 0.999 and np.mean(dist[k:] <= 1) >= 0.999
    assert_far_misses_are_tiny(Wn, ref["W_new"], dist, fmt, 0.1)
    assert_dx_close(dX, ref["dX_partial"], 6e-2)
    same = dist[:k] == 0
    cg, cr = o.decode_bf16(case.C()), o.decode_bf16(ref["comp_new"][:k])
    scale = np.maximum(np.abs(o.decode(ref["W_new"][:k], fmt)), 2.0**-9)
    assert np.quantile((np.abs(cg - cr) / scale)[same], 0.999) <= 2.0**-8
    # the mode is not the all-Kahan one: rows past the boundary equal the oracle's plain update
    plain = o.head_step(case.W0[k:], None, X, indptr, indices, 0.1, 3, 5, fmt, o.FLAG_SR, label_ids=np.arange(k, L))
    assert np.mean(np.abs(ordered(Wn[k:], fmt) - ordered(plain["W_new"], fmt)) <= 1) >= 0.999


@pytest.mark.parametrize("fmt,flags,B", [
    (o.E4M3, o.FLAG_SR | o.FLAG_KAHAN, 70),
    (o.E4M3, o.FLAG_SR, 300),
    (o.BF16, o.FLAG_KAHAN, 300),
    (o.BF16, o.FLAG_SR, 70),
])
def test_weight_decay(b, fmt, flags, B):
    """The L2 term g + wd*w in both update kernels (single-pass small-batch and 256 x 256 tiles),
    with a decay large enough to move many weights by itself."""
    L, d, chunk, wd, lr = 3 * 128 + 50, 256, 256, 0.1, 0.1
    case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.2, comp_std=2e-4, seed=16, weight_decay=wd)
    rng = np.random.default_rng(31)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    say(f"[weight decay] fmt={fmt} flags={flags} B={B} wd={wd}")
    dX, loss = case.step(X, indptr, indices, lr, 8, 2)
    ref = o.head_step(case.W0, case.C0, X, indptr, indices, lr, 8, 2, fmt, flags, weight_decay=wd)
    nowd = o.head_step(case.W0, case.C0, X, indptr, indices, lr, 8, 2, fmt, flags)
    Wn = case.W()
    dist = np.abs(ordered(Wn, fmt) - ordered(ref["W_new"], fmt))
    moved = float(np.mean(ref["W_new"] != nowd["W_new"]))
    say(f"   W': exact {np.mean(dist == 0):.5f}, within 1 ulp {np.mean(dist <= 1):.6f}; the decay changes {moved:.3f} of the codes")
    assert moved > 0.01
    assert np.mean(dist <= 1) >= 0.999
    assert_far_misses_are_tiny(Wn, ref["W_new"], dist, fmt, lr)
    assert_dx_close(dX, ref["dX_partial"], 6e-2 if fmt == o.E4M3 else 2e-2)


@pytest.mark.parametrize("fmt,flags,B,d,T", [
    (o.E4M3, o.FLAG_SR | o.FLAG_KAHAN, 300, 384, 64),
    (o.E4M3, o.FLAG_SR, 70, 256, 128),
    (o.E4M3, 0, 600, 256, 230),
    (o.BF16, o.FLAG_KAHAN, 300, 256, 26),
    (o.BF16, o.FLAG_SR, 70, 128, 200),
    (o.BF16, 0, 300, 384, 128),
    (o.E4M3, o.FLAG_SR | o.FLAG_KAHAN, 70, 512, 77),     # single-pass small-batch kernel with its masked tile copy
    (o.BF16, o.FLAG_SR, 100, 256, 128),                  # the same, BF16 weights
    (o.BF16, o.FLAG_KAHAN, 70, 256, 128),                # BF16 + compensation: no room for the copy, separate kernels
    (o.E4M3, 0, 40, 256, 200),
])
def test_classifier_dropout(b, fmt, flags, B, d, T):
    """Dropout on the weights inside the three products: the library regenerates the oracle's mask
    from (seed, step, element) in the logits, the input-gradient and the update kernel, for both
    logits tile sizes, a width with a half column tile, ragged label tails and several chunks.
    A mask that differed in one kernel, or a missing scale, would miss every bar here: the logits
    feed the loss and G, the input gradient sums masked weights, and the weight gradient of a
    dropped element is zero, so without rounding noise and compensation it must not move at all."""
    L, chunk, lr = 3 * 256 + 77, 512, 0.1
    case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.05, comp_std=2e-4, seed=23, dropout_p=T / 256)
    rng = np.random.default_rng(41)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    say(f"[dropout] fmt={fmt} flags={flags} B={B} d={d} T={T}")
    dX, loss = case.step(X, indptr, indices, lr, 77, 4)
    ref = o.head_step(case.W0, case.C0, X, indptr, indices, lr, 77, 4, fmt, flags, dropout=T)
    plain = o.head_step(case.W0, case.C0, X, indptr, indices, lr, 77, 4, fmt, flags)
    Wn = case.W()
    dist = np.abs(ordered(Wn, fmt) - ordered(ref["W_new"], fmt))
    e_dx, e_loss = rel_fro(dX, ref["dX_partial"]), abs(loss - ref["loss"]) / abs(ref["loss"])
    say(f"   W': exact {np.mean(dist == 0):.5f}, within 1 ulp {np.mean(dist <= 1):.6f};  dX rel-Fro {e_dx:.2e} "
        f"(no-dropout oracle is {rel_fro(plain['dX_partial'], ref['dX_partial']):.2e} away);  loss rel {e_loss:.2e}")
    assert rel_fro(plain["dX_partial"], ref["dX_partial"]) > 0.2        # the mask matters at this rate
    assert np.mean(dist <= 1) >= 0.999
    assert_far_misses_are_tiny(Wn, ref["W_new"], dist, fmt, lr)
    assert_dx_close(dX, ref["dX_partial"], 6e-2 if fmt == o.E4M3 else 2e-2)
    assert e_loss <= 2e-3
    if flags == 0:
        keep = o.dropout_keep(77, 4, np.arange(L * d, dtype=np.int64).reshape(L, d), T)
        assert np.array_equal(Wn[~keep], case.W0[~keep])
        assert np.any(Wn[keep] != case.W0[keep])
    # the mask is a function of the element, not of the chunking
    other = Case(b, L, d, fmt, 256, flags, B, w_std=0.05, comp_std=2e-4, seed=23, dropout_p=T / 256)
    other.step(X, indptr, indices, lr, 77, 4)
    assert np.array_equal(other.W(), Wn)
    with pytest.raises(b.ElmoError):
        case.head.step(dev(X), dev(indptr), dev(indices), lr, 77, 1 << 63)


@pytest.mark.parametrize("B,d,flags,L,chunk", [
    (70, 768, o.FLAG_SR | o.FLAG_KAHAN, 9 * 128 + 77, 512),     # 128-row padded batch, the width of the 3M-label head
    (128, 256, o.FLAG_SR, 2048 + 1, 1024),                       # full batch tile, one label past a tile boundary
    (33, 512, o.FLAG_KAHAN, 700, 384),                           # 64-row padded batch
    (64, 1536, 0, 300, 256),                                     # 64 rows x 1536 columns: the largest resident input
    (5, 256, o.FLAG_SR, 40, 128),                                # fewer labels than one strip group
])
def test_small_batch_logits_without_loss(b, B, d, flags, L, chunk):
    """A step that asks for no loss value (what the benchmark times) runs the logits kernel built
    without the loss terms.  Checked against the oracle like every step, and bit for bit against
    the same step with a loss output: both accumulate every logit over K in the same order, so G
    and the updated weights must agree.  Small batches (padded to 64 or 128 rows), E4M3 weights,
    crowded first label bins, ragged label counts."""
    rng = np.random.default_rng(91)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.3).draw_csr(rng, B, "lognormal5")    # steep: the first bins are crowded
    say(f"[stream logits] B={B} d={d} flags={flags} L={L} chunk={chunk} nnz={len(indices)}")
    case = Case(b, L, d, o.E4M3, chunk, flags, B, w_std=0.05, comp_std=2e-4, seed=92)
    check_step(case, X, indptr, indices, 0.1, 11, 3, 6e-2, want_loss=False)
    other = Case(b, L, d, o.E4M3, chunk, flags, B, w_std=0.05, comp_std=2e-4, seed=92)
    dX2, _ = other.step(X, indptr, indices, 0.1, 11, 3, want_loss=True)
    assert np.array_equal(other.W(), case.W())
    if flags & o.FLAG_KAHAN:
        assert np.array_equal(other.C(), case.C())


def test_many_batch_tiles(b):
    """A batch of 1100 rows: five 256-row batch tiles (the last one mostly padding), so the
    input-gradient partials are spread over several label slices per tile and the finalise
    kernel sums them."""
    L, d, B, chunk = 600, 128, 1100, 384
    case = Case(b, L, d, o.E4M3, chunk, o.FLAG_SR | o.FLAG_KAHAN, B, w_std=0.05, seed=18)
    rng = np.random.default_rng(19)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "fixed5")
    say(f"[many batch tiles] L={L} d={d} B={B}")
    check_step(case, X, indptr, indices, 0.02, 4, 1, 6e-2)


def test_same_operand_error_is_at_bf16_roundoff(b):
    """Sharper than the contract: G is held in BF16 (unit roundoff 2^-9), so dX should agree with
    the FP64 oracle to a few 1e-3 when both start from the same bits."""
    L, d, B = 2048, 256, 128
    case = Case(b, L, d, o.E4M3, 1024, o.FLAG_SR, B, w_std=0.05)
    rng = np.random.default_rng(8)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "fixed5")
    say("[same-operand] E4M3 L=2048 d=256 B=128")
    dX, _ = case.step(X, indptr, indices, 0.05, 1, 1)
    ref = o.head_step(case.W0, None, X, indptr, indices, 0.05, 1, 1, o.E4M3, o.FLAG_SR)
    assert_dx_close(dX, ref["dX_partial"], 6e-2)


@pytest.mark.parametrize("fmt,flags,B", [
    (o.E4M3, o.FLAG_SR | o.FLAG_KAHAN, 256), (o.E4M3, o.FLAG_SR | o.FLAG_KAHAN, 96), (o.BF16, o.FLAG_SR, 256), (o.BF16, o.FLAG_KAHAN, 96)])
def test_which_logit_gradient_the_kernels_compute(b, fmt, flags, B):
    """The logit gradient G = sigmoid(Z) - Y is held in 16 bits (Section 4.4 keeps the per-chunk
    logit-gradient buffer in 16 bits for BF16 and FP8 training; Algorithm 1 forms sigmoid and the
    "-1" in that buffer), so the oracle rounds its FP64 G once to BF16.  This test shows what that
    reading is worth: the same GPU step is compared with the oracle as it stands and with the oracle
    that keeps G in FP64 (g_exact).  The kernels must match the first at least as well as the second;
    the figures of both are printed for the record."""
    L, d, chunk, lr = 4096 + 77, 256, 1024, 0.05
    case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.02, seed=71)
    rng = np.random.default_rng(72)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.05).draw_csr(rng, B, "poisson7")
    dX, _ = case.step(X, indptr, indices, lr, 5, 3)
    Wn = case.W()
    out = {}
    for name, exact in (("G rounded to BF16", False), ("G kept in FP64", True)):
        ref = o.head_step(case.W0, case.C0, X, indptr, indices, lr, 5, 3, fmt, flags, g_exact=exact)
        dist = np.abs(ordered(Wn, fmt) - ordered(ref["W_new"], fmt))
        out[exact] = (float(np.mean(dist == 0)), float(np.mean(dist <= 1)), rel_fro(dX, ref["dX_partial"]))
        say(f"[G reading] fmt={fmt} flags={flags} B={B}  oracle with {name}: W' exact {out[exact][0]:.5f}, "
            f"within 1 ulp {out[exact][1]:.6f}, dX rel-Fro {out[exact][2]:.2e}")
    assert out[False][1] >= 0.999
    assert out[False][0] >= out[True][0] and out[False][2] <= out[True][2] + 1e-4


def test_weights_do_not_depend_on_chunk_and_steps_repeat(b):
    """Chunk invariance: identical updated weights for any chunk size at fixed (seed, step);
    same call twice from the same state gives the same bits; another step index does not."""
    L, d, B = 1000, 256, 96
    rng = np.random.default_rng(2)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "fixed5")
    flags = o.FLAG_SR | o.FLAG_KAHAN
    outs = []
    for chunk in (128, 384, 1024, 100, 1, 777):         # any positive chunk: a pass takes the next multiple of 128 labels
        case = Case(b, L, d, o.E4M3, chunk, flags, B, w_std=0.05, seed=1)
        say(f"[chunk-invariance] chunk={chunk}")
        dX, _ = case.step(X, indptr, indices, 0.05, 9, 4)
        outs.append((case.W(), case.C(), dX))
    for W, C, dX in outs[1:]:
        assert np.array_equal(W, outs[0][0]) and np.array_equal(C, outs[0][1])
        assert rel_fro(dX, outs[0][2]) < 1e-2
    case = Case(b, L, d, o.E4M3, 384, flags, B, w_std=0.05, seed=1)
    case.step(X, indptr, indices, 0.05, 9, 4)
    assert np.array_equal(case.W(), outs[0][0])
    case = Case(b, L, d, o.E4M3, 384, flags, B, w_std=0.05, seed=1)
    case.step(X, indptr, indices, 0.05, 9, 5)
    assert not np.array_equal(case.W(), outs[0][0])


def test_step_replays_bit_identically_from_a_hip_graph(b):
    """A training step only enqueues kernels on the caller's stream (no allocation, no memset node,
    no host synchronisation without ELMO_VALIDATE), so it can be captured: three replays of a
    captured step, with eager work and synchronisations between them, leave the same weights,
    compensation, input gradient and loss as three eager calls with the same arguments."""
    L, d, B, chunk = 3 * 256 + 77, 256, 300, 512
    fmt, flags = o.E4M3, o.FLAG_SR | o.FLAG_KAHAN
    rng = np.random.default_rng(51)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    Xd, ip, ix = dev(X), dev(indptr), dev(indices)
    results = []
    for mode in ("eager", "graph"):
        case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.05, comp_std=2e-4, seed=33)
        dX = torch.zeros(X.shape, dtype=torch.int16, device=DEV)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        case.head.step(Xd, ip, ix, 0.1, 9, 0, dX, loss)            # warm-up: one-time kernel attributes
        torch.cuda.synchronize()
        case.load(case.W0, case.C0)
        side = torch.cuda.Stream()
        graph = None
        if mode == "graph":
            graph = torch.cuda.CUDAGraph()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.graph(graph, stream=side):
                case.head.step(Xd, ip, ix, 0.1, 9, 4, dX, loss, torch.cuda.current_stream())
            torch.cuda.synchronize()
            case.load(case.W0, case.C0)                            # capture does not run the step
        snaps = []
        for rep in range(3):
            if graph is not None:
                graph.replay()
            else:
                case.head.step(Xd, ip, ix, 0.1, 9, 4, dX, loss)
            torch.cuda.synchronize()
            scratch = torch.randn(1 << 20, device=DEV).sum().item()   # unrelated eager work between replays
            snaps.append((case.W().copy(), case.C().copy(), host_u16(dX).copy(), float(loss.item())))
        results.append(snaps)
    say("[graph] three replays against three eager steps")
    for rep in range(3):
        for a, g_ in zip(results[0][rep][:3], results[1][rep][:3]):
            assert np.array_equal(a, g_), f"replay {rep} differs from the eager step"
        assert results[0][rep][3] == results[1][rep][3]
    assert not np.array_equal(results[0][0][0], results[0][2][0])     # the weights do move from replay to replay


def test_rne_cancels_tiny_updates_bit_identically(b):
    """Section 4.1: with nearest rounding an update below half a spacing leaves W untouched."""
    L, d, B = 512, 128, 32
    case = Case(b, L, d, o.BF16, 256, 0, B, w_std=0.3)
    rng = np.random.default_rng(4)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "fixed5")
    say("[rne-cancel]")
    case.step(X, indptr, indices, 1e-7, 0, 0, want_dx=False, want_loss=False)
    W = case.W()
    big = np.abs(o.decode_bf16(case.W0)) > 1e-2
    assert np.array_equal(W[big], case.W0[big])


def test_degenerate_inputs(b):
    """B = 1, a batch without positives, fewer labels than one tile, zero weights (closed form)."""
    L, d = 100, 128
    case = Case(b, L, d, o.BF16, 128, o.FLAG_SR, 4, max_nnz=16)
    rng = np.random.default_rng(6)
    X = synth.make_x(rng, 1, d)
    say("[degenerate] B=1, one positive")
    check_step(case, X, np.array([0, 1], np.int32), np.array([99], np.int32), 0.05, 0, 0, 2e-2)
    say("[degenerate] no positives at all")
    X = synth.make_x(rng, 3, d)
    check_step(case, X, np.zeros(4, np.int32), np.zeros(0, np.int32), 0.05, 0, 1, 2e-2)
    say("[degenerate] zero weights: dX = 0, loss = B L ln 2")
    case.load(np.zeros((L, d), np.uint16), None)
    dX, loss = case.step(X, np.array([0, 1, 1, 2], np.int32), np.array([5, 7], np.int32), 0.05, 0, 2)
    assert np.all(dX == 0)
    assert abs(loss - 3 * L * np.log(2.0)) < 1e-3 * 3 * L


def test_label_index_with_long_rows_crowded_bins_and_far_labels(b):
    """The per-step label index (positives regrouped by 128-label bin): a row with 300 positives (more
    than a thread keeps in registers between the index's two phases), 40 rows that all name the
    same few head labels (one crowded bin), and labels beyond the range that is counted in LDS
    first (ids >= 262144).  Every positive must arrive as exactly one "-1" in G: checked through
    the weight rows of the touched labels, the input gradient and the loss."""
    L, d, B, chunk, lr = 270000, 128, 70, 65536, 0.1
    fmt, flags = o.BF16, 0
    case = Case(b, L, d, fmt, chunk, flags, B, max_nnz=4096, w_std=0.05, seed=31)
    rng = np.random.default_rng(77)
    X = synth.make_x(rng, B, d)
    rows = []
    rows.append(np.unique(np.concatenate([rng.choice(400, 200, replace=False), rng.choice(np.arange(262144, L), 100, replace=False)])))
    for i in range(1, 41):
        rows.append(np.array([0, 1, 2, 3, 127, 128, 262144 + i, L - 1]))
    for i in range(41, B):
        rows.append(np.unique(rng.integers(0, L, size=rng.integers(0, 9))))
    indptr = np.zeros(B + 1, np.int32)
    indptr[1:] = np.cumsum([len(r) for r in rows])
    indices = np.concatenate(rows).astype(np.int32)
    say(f"[label index] L={L} B={B} nnz={len(indices)} longest row {max(len(r) for r in rows)}")
    dX, loss = case.step(X, indptr, indices, lr, 5, 1)
    touched = np.unique(indices)
    sample = np.unique(np.concatenate([touched, rng.integers(0, L, 4000)]))
    ref = o.head_step(case.W0[sample], None, X, indptr, indices, lr, 5, 1, fmt, flags, label_ids=sample)
    Wn = case.W()[sample]
    dist = np.abs(ordered(Wn, fmt) - ordered(ref["W_new"], fmt))
    say(f"   W' on {len(sample)} label rows ({len(touched)} with positives): within 1 ulp {np.mean(dist <= 1):.6f}")
    assert np.mean(dist <= 1) >= 0.999
    assert_far_misses_are_tiny(Wn, ref["W_new"], dist, fmt, lr)
    # rows with positives move against X; a lost or doubled "-1" would change them by lr * |x| ~ 1e-2
    hot = np.isin(sample, touched)
    assert np.max(np.abs(o.decode(Wn[hot], fmt) - o.decode(ref["W_new"][hot], fmt))) < 1e-3
    dX_ref, Z = o.input_gradient_rows(case.W0, X, indptr, indices, fmt, np.arange(B))
    assert_dx_close(dX, dX_ref, 2e-2)
    Y = o.csr_to_dense(indptr, indices, L)
    assert abs(loss - o.bce_loss(Z, Y)) / o.bce_loss(Z, Y) < 2e-3


@pytest.mark.parametrize("fmt,flags", [(o.E4M3, o.FLAG_SR | o.FLAG_KAHAN), (o.E4M3, 0), (o.BF16, o.FLAG_SR)])
def test_saturating_updates_clip_to_the_largest_finite_value(b, fmt, flags):
    """A learning rate so large that most updates leave the format's range: the result clips to the
    largest finite value on both sides (no NaN, no infinity), rounding mode and compensation included."""
    L, d, B, chunk = 3 * 128 + 50, 256, 70, 256
    lr = 3.0e5 if fmt == o.E4M3 else 3.0e38     # BF16: products around the top of the FP32 range, some beyond it
    case = Case(b, L, d, fmt, chunk, flags, B, w_std=0.05, seed=61)
    rng = np.random.default_rng(63)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    say(f"[saturation] fmt={fmt} flags={flags} lr={lr:g}")
    with np.errstate(over="ignore", invalid="ignore"):
        ref = o.head_step(case.W0, case.C0, X, indptr, indices, lr, 2, 0, fmt, flags)
    case.step(X, indptr, indices, lr, 2, 0)
    Wn = case.W()
    top = 0x7E if fmt == o.E4M3 else 0x7F7F
    mag = (Wn & 0x7F) if fmt == o.E4M3 else (Wn & 0x7FFF)
    clipped = float(np.mean(mag == top))
    say(f"   {clipped:.3f} of the weights sit at the largest finite value")
    assert np.all(mag <= top) and (clipped > 0.5 or fmt == o.BF16)      # finite everywhere; E4M3 mostly at +-448
    dist = np.abs(ordered(Wn, fmt) - ordered(ref["W_new"], fmt))
    # the sign of a clipped weight is the sign of a large FP32 sum, which both sides agree on
    # except where the gradient itself is within rounding of zero
    assert np.mean(dist <= 1) >= 0.999


def test_validation_flag_reports_bad_labels_on_the_next_call(b):
    """Bad label ids are caught by the kernels' own bounds checks (nothing faults) and surface
    as error -4 on the following call."""
    L, d = 300, 128
    head = b.Head(L, d, b.ELMO_BF16, 128, b.ELMO_VALIDATE, 4, 16)
    X = dev(synth.make_x(np.random.default_rng(0), 2, d))
    say("[validate] out-of-range label id")
    head.step(X, dev(np.array([0, 1, 2], np.int32)), dev(np.array([5, 300], np.int32)), 0.05, 0, 0)
    torch.cuda.synchronize()
    with pytest.raises(b.ElmoError) as e:
        head.step(X, dev(np.array([0, 1, 2], np.int32)), dev(np.array([5, 6], np.int32)), 0.05, 0, 1)
    assert e.value.code == -4
    head.step(X, dev(np.array([0, 1, 2], np.int32)), dev(np.array([5, 6], np.int32)), 0.05, 0, 1)
    torch.cuda.synchronize()
    head.step(X, dev(np.array([0, 1, 2], np.int32)), dev(np.array([5, 6], np.int32)), 0.05, 0, 2)
    torch.cuda.synchronize()
    with pytest.raises(b.ElmoError) as e:                       # B > max_B is refused on the host
        b.elmo_head_step(head.h, X, 5, dev(np.array([0, 1], np.int32)), None, 0, 0.05, 0, 0)
    assert e.value.code == -1


# --------------------------------------------------------------------------------- sampled checks at scale
def _sample_labels(L, chunk, indices, rng, n_random):
    ids = [np.unique(indices), np.arange(max(0, L - 300), L)]
    for c0 in range(0, L, chunk):
        ids.append(np.array([c0, min(L, c0 + chunk) - 1]))
    ids.append(rng.integers(0, L, size=n_random))
    return np.unique(np.concatenate(ids).astype(np.int64))


def _init_on_device(b, head, cfg, seed=0):
    """W0 ~ N(0, std) drawn on the device in slices and rounded to the storage format by the
    library's own nearest-even kernel (whose bit-exactness is tested above)."""
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    W = head.weights()
    rows = 65536
    for l0 in range(0, cfg.L, rows):
        l1 = min(cfg.L, l0 + rows)
        f = torch.randn((l1 - l0) * cfg.d, device=DEV, generator=g) * cfg.w_std
        b.elmo_quantize(f, f.numel(), cfg.fmt, 0, 0, 0, 0, W[l0:l1])
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,dx_rows", [("mid", 16), ("large", 16), ("xl", 16)])
def test_full_size_configs_on_samples(b, name, dx_rows):
    """Benchmark configurations 2-4 at full size in the launch configuration the benchmark times.
    Labels are independent given X, so the oracle evaluates a label sample exactly (all in-batch
    positives, chunk-boundary rows, the ragged tail, random rows) and a few full rows of dX."""
    _full_size_check(b, synth.CONFIGS[name], name, dx_rows, 2)


@pytest.mark.parametrize("B,chunk,kahan,dx_rows", [
    (128, 262144, True, 16), (128, 65536, False, 16), (32, 65536, True, 16), (32, 262144, False, 16),
    (4096, 65536, False, 16), (4096, 262144, True, 16)])
def test_xl_sweep_points_on_samples(b, B, chunk, kahan, dx_rows):
    """Benchmark configuration 5 (the bandwidth-regime sweep at 3M labels) at full size, in the launch
    configurations the benchmark times: all six (batch, chunk) points -- the small-batch kernels at
    B = 128 and B = 32, the 256 x 256-tile kernels with 16 batch tiles at B = 4096 -- with the
    compensation buffer on one chunk size of each batch and off on the other."""
    cfg = synth.xl_sweep(B, chunk, kahan)
    _full_size_check(b, cfg, cfg.name, dx_rows, 1)


def test_xl_config_step_after_twenty_unchecked_steps(b):
    """Benchmark configuration 4 runs 20 steps: the first 19 are only run (fresh batch each, as in the
    benchmark), the 20th is checked against the oracle started from the device state before it --
    what an error that builds up in the reused workspace or the compensation would break."""
    _full_size_check(b, synth.CONFIGS["xl"], "xl after 19 steps", 2, 1, unchecked=19)


def _full_size_check(b, cfg, name, dx_rows, steps, unchecked=0):
    tol = 6e-2 if cfg.fmt == o.E4M3 else 2e-2
    say(f"[{name}] L={cfg.L} d={cfg.d} B={cfg.B} chunk={cfg.chunk} fmt={cfg.fmt} flags={cfg.flags}: init")
    head = b.Head(cfg.L, cfg.d, cfg.fmt, cfg.chunk, cfg.flags, cfg.B, 64 * cfg.B)
    _init_on_device(b, head, cfg)
    zipf = synth.ZipfLabels(cfg.L, cfg.zipf_s)
    rng = np.random.default_rng(1)
    for step in range(unchecked):
        X, indptr, indices = synth.make_batch(cfg, step, zipf)
        head.step(dev(X), dev(indptr), dev(indices), cfg.lr, 0, step,
                  torch.zeros(X.shape, dtype=torch.int16, device=DEV), None)
    torch.cuda.synchronize()
    for step in range(unchecked, unchecked + steps):   # a second step starts from non-zero compensation
        X, indptr, indices = synth.make_batch(cfg, step, zipf)
        ids = _sample_labels(cfg.L, cfg.chunk, indices, rng, 4096)
        idt = torch.from_numpy(ids).to(DEV)
        Wb = head.weights()[idt].cpu().numpy()
        Wb = Wb.view(np.uint16) if cfg.fmt == o.BF16 else Wb
        Cb = host_u16(head.compensation()[idt]) if head.comp is not None else None
        rows = np.sort(rng.choice(cfg.B, size=min(dx_rows, cfg.B), replace=False))
        W_all = None
        if step == unchecked:
            W_all = head.weights().cpu().numpy()
            W_all = W_all.view(np.uint16) if cfg.fmt == o.BF16 else W_all
        Xd, ip, ix = dev(X), dev(indptr), dev(indices)
        dX = torch.zeros(X.shape, dtype=torch.int16, device=DEV)
        loss = torch.zeros(1, dtype=torch.float32, device=DEV)
        say(f"[{name}] step {step}: nnz={len(indices)}, {len(ids)} sampled labels, GPU step")
        head.step(Xd, ip, ix, cfg.lr, 0, step, dX, loss)
        torch.cuda.synchronize()
        say(f"[{name}] step {step}: oracle on the label sample")
        ref = o.head_step(Wb, Cb, X, indptr, indices, cfg.lr, 0, step, cfg.fmt, cfg.flags, label_ids=ids)
        Wn = head.weights()[idt].cpu().numpy()
        Wn = Wn.view(np.uint16) if cfg.fmt == o.BF16 else Wn
        dist = np.abs(ordered(Wn, cfg.fmt) - ordered(ref["W_new"], cfg.fmt))
        say(f"   W' sample: exact {np.mean(dist == 0):.5f}, within 1 ulp {np.mean(dist <= 1):.6f}, max {dist.max()}")
        assert np.mean(dist <= 1) >= 0.999
        assert_far_misses_are_tiny(Wn, ref["W_new"], dist, cfg.fmt, cfg.lr)
        if Cb is not None:
            cg = o.decode_bf16(host_u16(head.compensation()[idt]))
            same = dist == 0
            scale = np.maximum(np.abs(o.decode(ref["W_new"], cfg.fmt)), 2.0**-9)
            err = (np.abs(cg - o.decode_bf16(ref["comp_new"])) / scale)[same]
            assert np.quantile(err, 0.999) <= 2.0**-8
        if W_all is not None:
            say(f"[{name}] step {step}: oracle dX for rows {rows.tolist()} over all labels")
            dX_ref, _ = o.input_gradient_rows(W_all, X, indptr, indices, cfg.fmt, rows)
            got = o.decode_bf16(host_u16(dX))[rows]
            assert_dx_close(got, dX_ref, tol, f"dX rows (loss {loss.item():.6g})")
            assert np.isfinite(loss.item()) and loss.item() > 0
    head.close()


# --------------------------------------------------------------------------------- top-k
# Scores are FP32 sums of exact products (E4M3 x E4M3 and BF16 x BF16 products fit FP32), so they
# differ from the FP64 logits by the summation rounding only: at most d * 2^-24 of the sum of the
# terms' magnitudes; measured at most 2e-7 of the largest score.
TOPK_TOL = 1e-5


def assert_topk_row(idx_row, sc_row, z_row, ref_sc_row, eps, L):
    """One query row against the oracle's logits z_row over all L labels.  Several answers are right
    when scores tie to within rounding, so: what is unique -- the sorted scores -- must equal the
    oracle's k best to eps; every returned id must be valid (distinct, in range, reported with its own
    logit, scoring at least the oracle's k-th value - eps); and the set must be complete: no label
    whose logit beats the weakest returned one by more than eps may be missing (a result that drops
    the true best label and returns the (k+1)-th instead fails here)."""
    k = len(idx_row)
    assert len(set(idx_row.tolist())) == k and idx_row.min() >= 0 and idx_row.max() < L
    assert np.all(np.diff(sc_row) <= 0)
    got_z = z_row[idx_row]
    assert np.all(np.abs(sc_row - got_z) <= eps), "a score is not its label's logit"
    assert np.all(got_z >= ref_sc_row[-1] - eps), "a returned label scores below the k-th best"
    assert np.all(np.abs(sc_row - ref_sc_row) <= eps), "the sorted scores are not the k best"
    above = np.nonzero(z_row > got_z.min() + eps)[0]
    missing = np.setdiff1d(above, idx_row)
    assert missing.size == 0, f"labels {missing[:5].tolist()} beat the weakest returned score and are absent"


def _check_topk(b, head, Wbits, X, k, fmt, tol=TOPK_TOL):
    B = X.shape[0]
    idx = torch.zeros((B, k), dtype=torch.int32, device=DEV)
    sc = torch.zeros((B, k), dtype=torch.float32, device=DEV)
    head.topk(dev(X), k, idx, sc)
    torch.cuda.synchronize()
    idx, sc = idx.cpu().numpy(), sc.cpu().numpy().astype(np.float64)
    Z = o.logits(Wbits, X, fmt)
    ref_idx, ref_sc = o.topk(Z, k)
    exact = float(np.mean(idx == ref_idx))
    eps = tol * max(np.abs(Z).max(), 1e-30)
    for i in range(B):
        assert_topk_row(idx[i], sc[i], Z[i], ref_sc[i], eps, Wbits.shape[0])
    worst = float(np.abs(sc - np.take_along_axis(Z, idx.astype(np.int64), axis=1)).max())
    say(f"   top-{k}: ids identical to the FP64 order in {exact:.4f} of the slots; largest score error {worst:.2e} (eps {eps:.2e})")
    return exact


@pytest.mark.parametrize("fmt", [o.BF16, o.E4M3])
def test_topk_small_brute_force(b, fmt):
    L, d, B = 3000 + 17, 256, 70
    case = Case(b, L, d, fmt, 1024, 0, B, w_std=0.05, seed=12)
    X = synth.make_x(np.random.default_rng(1), B, d)
    for k in (1, 5, 100, 128):
        say(f"[topk-small] fmt={fmt} k={k}")
        _check_topk(b, case.head, case.W0, X, k, fmt)


@pytest.mark.parametrize("fmt", [o.E4M3, o.BF16])
def test_topk_one_slab_per_tile_and_several_batch_tiles(b, fmt):
    """d = 128: an E4M3 tile is a single 128-byte K slab, so the kernel that keeps its ring running from
    tile to tile changes tile at every slab (thresholds of the next tile's rows fetched a tile ahead);
    300 queries are two batch tiles, the second ragged; 9000 + 5 labels are the first level, two
    more levels (both in the form for levels where many scores pass) and a ragged last label tile;
    k = 100 and a second page (k = 130)."""
    L, d, B = 9000 + 5, 128, 300
    case = Case(b, L, d, fmt, 4096, 0, B, w_std=0.05, seed=23)
    X = synth.make_x(np.random.default_rng(5), B, d)
    for k in (100, 130):
        say(f"[topk-one-slab] fmt={fmt} k={k}")
        _check_topk(b, case.head, case.W0, X, k, fmt)


def test_topk_passes_collected_per_workgroup_over_several_label_tiles(b):
    """Three batch tiles (600 queries) and a last level of 93 label tiles: more tiles than one workgroup
    per CU, so the workgroups of that level walk one or two label tiles of one batch tile (a grid of 255,
    the multiple of three below 256) and hands the passes it collected in LDS to the rows' lists at its
    end; with k = 20 few scores pass per row, with k = 60 (the largest k for which that level still
    takes the sparse form) a few rows fill their eight LDS entries and append the rest directly.  Both
    against the oracle's full sort."""
    L, d, B = 40000 + 3, 128, 600
    case = Case(b, L, d, o.E4M3, 8192, 0, B, w_std=0.05, seed=29)
    X = synth.make_x(np.random.default_rng(6), B, d)
    for k in (20, 60):
        say(f"[topk-collect] k={k}")
        _check_topk(b, case.head, case.W0, X, k, o.E4M3)


@pytest.mark.parametrize("fmt,L,B,ks", [(o.E4M3, 3000 + 17, 70, (129, 300, 500)), (o.BF16, 300, 9, (256, 300)), (o.E4M3, 131, 3, (131,))])
def test_topk_beyond_one_page(b, fmt, L, B, ks):
    """k above 128 comes in pages of 128 entries, every page one more sweep that admits only what
    ranks strictly after the page before: against the oracle's full sort, up to k = L (the whole
    ranking of every row), with a last page of a single entry (k = 129) and a head smaller than two pages."""
    d = 256
    case = Case(b, L, d, fmt, 1024, 0, B, w_std=0.05, seed=19)
    X = synth.make_x(np.random.default_rng(4), B, d)
    for k in ks:
        say(f"[topk-pages] fmt={fmt} L={L} B={B} k={k}")
        _check_topk(b, case.head, case.W0, X, k, fmt)
    with pytest.raises(b.ElmoError):
        case.head.topk(dev(X), L + 1, None, None)


def test_topk_pages_with_tied_scores_and_the_unbounded_path(b):
    """Pages across ties and across the overflow path: all-zero weights (every score ties, the answer
    is ids 0..k-1 whatever the page boundaries cut through) and scores rising with the label id (every
    page overflows the fast path's candidate lists)."""
    L, d, B, k = 1000, 128, 5, 300
    case = Case(b, L, d, o.BF16, 512, 0, B)
    case.load(np.zeros((L, d), np.uint16), None)
    idx = torch.zeros((B, k), dtype=torch.int32, device=DEV)
    sc = torch.ones((B, k), dtype=torch.float32, device=DEV)
    say("[topk-pages] ties")
    case.head.topk(dev(synth.make_x(np.random.default_rng(0), B, d)), k, idx, sc)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), np.tile(np.arange(k), (B, 1))) and np.all(sc.cpu().numpy() == 0)
    L, d, B, k = 40000, 128, 9, 260
    rng = np.random.default_rng(5)
    X = synth.make_x(rng, B, d)
    u = o.decode_bf16(X).mean(axis=0)
    u /= np.linalg.norm(u)
    ramp = np.linspace(0.0, 2.0, L)[:, None] * u[None, :] + rng.standard_normal((L, d)) * 1e-3
    case = Case(b, L, d, o.BF16, 4096, 0, B)
    W = o.round_bf16(ramp.astype(np.float32))
    case.load(W, None)
    say("[topk-pages] rising scores, k=260")
    assert _check_topk(b, case.head, W, X, k, o.BF16) > 0.9


def test_topk_mid_size_k500(b):
    """k = 500 over the Mid head's 131072 labels (four pages)."""
    cfg = synth.CONFIGS["mid"]
    head = b.Head(cfg.L, cfg.d, cfg.fmt, cfg.chunk, 0, 64, 64)
    _init_on_device(b, head, cfg)
    W = head.weights().cpu().numpy().view(np.uint16)
    X = synth.make_x(np.random.default_rng(3), 48, cfg.d)
    say("[topk-mid] L=131072 B=48 k=500")
    _check_topk(b, head, W, X, 500, cfg.fmt)
    head.close()


def test_wide_head_on_the_small_batch_path(b):
    """An embedding wider than 65536 columns with a small batch: more column blocks than the 256
    workgroups the single-pass kernel spreads over label groups, so one label group does all tiles."""
    L, d, B = 40, 65536 + 256, 4
    case = Case(b, L, d, o.E4M3, 128, o.FLAG_SR, B, max_nnz=64, w_std=0.01, seed=5)
    rng = np.random.default_rng(6)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "fixed5")
    say(f"[wide head] L={L} d={d} B={B}")
    check_step(case, X, indptr, indices, 0.05, 1, 0, 6e-2)


def test_topk_ties_prefer_smaller_ids(b):
    """All-zero weights: every logit ties at 0, so the answer is ids 0..k-1 in order."""
    L, d, B, k = 1000, 128, 5, 10
    case = Case(b, L, d, o.BF16, 512, 0, B)
    case.load(np.zeros((L, d), np.uint16), None)
    idx = torch.zeros((B, k), dtype=torch.int32, device=DEV)
    sc = torch.ones((B, k), dtype=torch.float32, device=DEV)
    say("[topk-ties]")
    case.head.topk(dev(synth.make_x(np.random.default_rng(0), B, d)), k, idx, sc)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), np.tile(np.arange(k), (B, 1))) and np.all(sc.cpu().numpy() == 0)


def test_topk_rising_scores_take_the_unbounded_path(b):
    """Scores that rise with the label id beat every threshold taken from earlier labels, so the
    per-row candidate lists of the fast path overflow and the capacity-free path must answer."""
    L, d, B, k = 40000, 128, 9, 20
    rng = np.random.default_rng(5)
    X = synth.make_x(rng, B, d)
    u = o.decode_bf16(X).mean(axis=0)
    u /= np.linalg.norm(u)
    ramp = np.linspace(0.0, 2.0, L)[:, None] * u[None, :] + rng.standard_normal((L, d)) * 1e-3
    case = Case(b, L, d, o.BF16, 4096, 0, B)
    W = o.round_bf16(ramp.astype(np.float32))
    case.load(W, None)
    say("[topk-rising] L=40000 B=9 k=20")
    exact = _check_topk(b, case.head, W, X, k, o.BF16)
    assert exact > 0.9


def test_precision_hits_bit_exact(b):
    """P@k numerators on the device against the oracle's count, on the head's own top-k and on
    hand-made predictions that contain every true label (ids up front)."""
    L, d, B, k = 3000, 256, 200, 10
    case = Case(b, L, d, o.E4M3, 1024, 0, B, w_std=0.05, seed=14)
    rng = np.random.default_rng(15)
    X = synth.make_x(rng, B, d)
    indptr, indices = synth.ZipfLabels(L, 1.0).draw_csr(rng, B, "lognormal5")
    idx = torch.zeros((B, k), dtype=torch.int32, device=DEV)
    case.head.topk(dev(X), k, idx, None)
    hits = torch.zeros(k, dtype=torch.int64, device=DEV)
    b.elmo_precision_hits(idx, B, k, dev(indptr), dev(indices), hits)
    torch.cuda.synchronize()
    want = o.precision_hits(idx.cpu().numpy(), indptr, indices)
    say(f"[P@k] hits {hits.cpu().numpy().tolist()}")
    np.testing.assert_array_equal(hits.cpu().numpy(), want)
    made = np.full((B, k), L - 1, dtype=np.int32)          # the true labels first, then a filler id
    for i in range(B):
        t = indices[indptr[i]:indptr[i + 1]][:k]
        made[i, :len(t)] = t
    b.elmo_precision_hits(dev(made), B, k, dev(indptr), dev(indices), hits)
    torch.cuda.synchronize()
    want = o.precision_hits(made, indptr, indices)
    assert want[0] == B                                    # every row has a positive: P@1 = 1
    np.testing.assert_array_equal(hits.cpu().numpy(), want)


def test_topk_mid_size(b):
    cfg = synth.CONFIGS["mid"]
    head = b.Head(cfg.L, cfg.d, cfg.fmt, cfg.chunk, 0, 64, 64)
    _init_on_device(b, head, cfg)
    W = head.weights().cpu().numpy().view(np.uint16)
    X = synth.make_x(np.random.default_rng(3), 64, cfg.d)
    say("[topk-mid] L=131072 B=64 k=100")
    _check_topk(b, head, W, X, 100, cfg.fmt)


def test_topk_xl_k100_on_sampled_queries(b):
    """Benchmark configuration 5, inference part: elmo_head_topk with k = 100 over all 3M logits for 1024
    queries.  Every row is checked for shape properties (distinct ids in range, scores sorted);
    sixteen sampled rows are checked against the oracle's logits over all labels (scores, validity
    and completeness of the returned set)."""
    cfg = synth.CONFIGS["xl"]
    B, k = 1024, 100
    head = b.Head(cfg.L, cfg.d, cfg.fmt, cfg.chunk, 0, B, 64)
    _init_on_device(b, head, cfg)
    X = synth.make_x(np.random.default_rng(9), B, cfg.d)
    idx = torch.zeros((B, k), dtype=torch.int32, device=DEV)
    sc = torch.zeros((B, k), dtype=torch.float32, device=DEV)
    say("[topk-xl] L=3000000 B=1024 k=100")
    head.topk(dev(X), k, idx, sc)
    torch.cuda.synchronize()
    idx, sc = idx.cpu().numpy(), sc.cpu().numpy().astype(np.float64)
    assert idx.min() >= 0 and idx.max() < cfg.L
    assert np.all(np.diff(sc, axis=1) <= 0)
    assert all(len(set(r.tolist())) == k for r in idx)
    rows = np.sort(np.random.default_rng(10).choice(B, size=16, replace=False))
    W = head.weights().cpu().numpy()
    Z = np.empty((len(rows), cfg.L))
    for l0 in range(0, cfg.L, 262144):
        Z[:, l0:l0 + 262144] = o.logits(W[l0:l0 + 262144], X[rows], cfg.fmt)
    ref_idx, ref_sc = o.topk(Z, k)
    eps = TOPK_TOL * np.abs(Z).max()
    for j, i in enumerate(rows):
        assert_topk_row(idx[i], sc[i], Z[j], ref_sc[j], eps, cfg.L)
    say(f"   ids identical to the FP64 order in {np.mean(idx[rows] == ref_idx):.4f} of the sampled slots")
    head.close()
