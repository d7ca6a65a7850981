"""CPU oracle for the ELMO classifier-head training step (TEST INFRASTRUCTURE ONLY).

This module is the slow, plain, FP64 statement of what the head's hot path computes.  It is
imported only by the tests, by the smoke check and by the benchmark's CPU-baseline leg.  It
shares no code, tables or constants with the HIP library and never calls it; the product path
never calls this module.

What is computed follows the paper (ELMO, arxiv 2510.11168):

* number formats and quantisation error                     -- Section 3 "Floating-point formats"
* stochastic rounding SR(x)                                  -- Section 3, Eq. (1)
* Kahan-compensated accumulation                             -- Section 3, the three-line recurrence
* classifier logit gradient  G = sigmoid(Z) - Y, InputGrad = G W, grad W = G^T X
                                                             -- Appendix "Background of Skipping
                                                                Loss Computation"
* order of operations of one head step (logits from the E4M3 cast of X, sigmoid, minus one at
  the positives, input gradient from the not-yet-updated weights, then the fused
  gradient + SGD + stochastic-rounding update with FP32 arithmetic)
                                                             -- Algorithm 1 and Section 4.3
* momentum-free SGD for the head                             -- Section 4.2
* Kahan compensation kept in BF16 for head weights           -- Appendix "Precision Recovery"
* top-k of the score vector and the P@k numerators          -- Appendix, definition of P@k
* compensation for the head labels only (kahan_rows)         -- Appendix "Precision Recovery"
* weight decay of the classifier                             -- Appendix, hyper-parameter table
* simulated (exponent, mantissa) formats                     -- Section 4.3 "8-Bit Training"
* dropout on the classifier weights inside the products     -- Appendix "Low-Memory Dropout for
                                                                Classifier"
* AdamW with Kahan-compensated BF16 parameters (encoder)     -- Section 4.1

Label chunking (Section 4.2) does not appear here: every label's logit, gradient row and weight
update depend only on that label's own weight row, so the chunked and unchunked results are the
same numbers and the oracle is written unchunked.

Readings taken where the paper is silent (each is repeated at the function that applies it):

* E4M3 is the OCP "FN" flavour (bias 7, largest finite 448, no infinities, one NaN code per
  sign); finite values beyond the largest finite value clip to it (the paper's "clipping error").
* BF16 likewise clips finite overflow to its largest finite value.
* Random numbers: Philox4x32-10 (Salmon et al., SC'11).  key = (seed low, seed high 32 bits);
  counter = (block low, block high, step low, step high) with block = e // 8 for the flat
  element index e = label * d + column of the whole [L, d] weight matrix.  The four output words
  hold eight 16-bit fields; element e uses field e % 8 (field f = word f // 2, low half first).
* The 16-bit field r decides the rounding by add-and-truncate on the magnitude: the 16 most
  significant dropped bits of |t| plus r carry into the kept bits or not.  For BF16 (16 dropped
  bits of an FP32 value) this is Eq. (1) exactly.  For E4M3 this DEPARTS from Eq. (1): 20 bits are
  dropped in the normal range, the field has 16, so the probability of rounding up is Eq. (1)'s
  rounded DOWN to a multiple of 2^-16 -- a bias of less than 2^-16 of a grid step toward zero per
  rounding (pinned exactly: over all 65536 fields the number that round up is floor(p 2^16)).
* Rounding acts on sign and magnitude separately; a result that rounds to zero keeps its sign.
* The weight gradient is summed over the batch with no 1/B factor (Algorithm 1, fuse_update).
* grad W uses the BF16 inputs X, the logits use the E4M3 cast of X (Algorithm 1).
* With both Kahan and SR enabled, SR is the rounding of s + y and the compensation captures the
  (random) rounding error; compensation is stored round-to-nearest-even in BF16.
* The FP32 update arithmetic is two separately rounded operations, lr * g then w - (lr * g).
* The logit gradient G is held in BF16: Section 4.4 keeps the per-chunk logit / logit-gradient
  buffer in 16 bits for BF16 and FP8 training alike, and Algorithm 1 forms sigmoid and the "-1" in
  that buffer.  Here Z stays FP64 and G = sigmoid(Z) - Y is rounded once, to nearest even, to
  BF16 before it enters the two products; both products then run in FP64.  `g_exact=True` skips
  that one rounding (used to pin the formulas by finite differences).
* Weight decay (the table only gives a value): the L2 term of plain SGD, g + wd*w in FP32, each
  operation rounded; absent (not merely zero) when wd = 0.
* Head labels are a prefix of the label ids (labels numbered by falling frequency).
* Kahan-AdamW: the paper defers to a library; taken here is textbook AdamW (decoupled decay,
  bias correction) in FP32 with every operation rounded once, the Kahan recurrence on the
  parameter, moments in BF16 (round to nearest) or FP32 (kahan_adamw).
* Classifier dropout: one keep bit per weight element and step (shared by the batch), from a
  second Philox stream; dropped with probability T/256, kept weights scaled by 256/(256-T); the
  masked weights serve logits and input gradient and mask the weight gradient (dropout_keep,
  head_step).

Parity pins: every function below is pinned by a CPU test against something other than itself
(published Philox vectors, torch's CPU casts, exhaustive enumeration of the random field,
closed forms, finite differences, brute force).  The one exception:

* training dynamics / end accuracy (P@k on the paper's datasets): parity unpinned -- the
  datasets and encoders are not available.
"""
from __future__ import annotations

import numpy as np

BF16 = 0
E4M3 = 1

FLAG_SR = 1
FLAG_KAHAN = 2

_U32 = np.uint64(0xFFFFFFFF)

# --------------------------------------------------------------------------------------------
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3")
# --------------------------------------------------------------------------------------------


def philox4x32_10(ctr, key):
    """Philox4x32 with 10 rounds.

    ctr: array [..., 4] of 32-bit words, key: array [..., 2] (broadcastable).  Returns uint32
    [..., 4].  Each round multiplies words 0 and 2 by the two Philox multipliers, and the new
    counter is (hi(m1*c2)^c1^k0, lo(m1*c2), hi(m0*c0)^c3^k1, lo(m0*c0)); the key is bumped by
    the two Weyl constants after every round.
    """
    ctr = np.asarray(ctr, dtype=np.uint64)
    key = np.asarray(key, dtype=np.uint64)
    c0, c1, c2, c3 = (ctr[..., i] & _U32 for i in range(4))
    k0, k1 = key[..., 0] & _U32, key[..., 1] & _U32
    m0 = np.uint64(0xD2511F53)
    m1 = np.uint64(0xCD9E8D57)
    w0 = np.uint64(0x9E3779B9)
    w1 = np.uint64(0xBB67AE85)
    s32 = np.uint64(32)
    for _ in range(10):
        p0 = m0 * c0
        p1 = m1 * c2
        c0, c1, c2, c3 = ((p1 >> s32) ^ c1 ^ k0) & _U32, p1 & _U32, ((p0 >> s32) ^ c3 ^ k1) & _U32, p0 & _U32
        k0 = (k0 + w0) & _U32
        k1 = (k1 + w1) & _U32
    out = np.stack(np.broadcast_arrays(c0, c1, c2, c3), axis=-1)
    return out.astype(np.uint32)


def sr_fields(seed: int, step: int, elem):
    """16-bit random field of each flat element index in `elem` (any integer array).

    Reading (paper names no generator): block = e // 8 is the low 64 bits of the Philox
    counter, the step is the high 64 bits, the seed is the key; field e % 8 of the 128 output
    bits, counted from the low half of word 0.
    """
    elem = np.asarray(elem, dtype=np.uint64)
    blk = elem >> np.uint64(3)
    fld = (elem & np.uint64(7)).astype(np.int64)
    ctr = np.stack(
        [
            blk & _U32,
            blk >> np.uint64(32),
            np.full(blk.shape, step & 0xFFFFFFFF, dtype=np.uint64),
            np.full(blk.shape, (step >> 32) & 0xFFFFFFFF, dtype=np.uint64),
        ],
        axis=-1,
    )
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint64)
    words = philox4x32_10(ctr, key).astype(np.uint64)
    w = np.take_along_axis(words, (fld >> 1)[..., None], axis=-1)[..., 0]
    return ((w >> (np.uint64(16) * (fld & 1).astype(np.uint64))) & np.uint64(0xFFFF)).astype(np.uint32)


def dropout_keep(seed: int, step: int, elem, threshold: int):
    """Keep mask (bool) of the classifier dropout for the flat weight-element indices `elem`
    (appendix "Low-Memory Dropout for Classifier": the weights are masked after they are loaded,
    before the matrix product, so no masked copy of W exists; the mask must therefore be a pure
    function of (seed, step, element)).

    Reading (the paper gives neither the generator nor the granularity): one mask per weight
    element and step, shared by all samples of the batch.  Philox4x32-10 with the seed as key and
    counter = (block low, block high, step low, step high | 2^31) for block = e // 16 -- the top
    counter bit keeps this stream apart from the rounding fields, which use steps below 2^63.
    The 128 output bits are sixteen bytes (byte b = bits [8 (b % 4), +8) of word b // 4);
    element e is kept iff byte e % 16 >= threshold, i.e. dropped with probability threshold / 256.
    """
    if not 0 <= threshold <= 255:
        raise ValueError("threshold must be in [0, 255]")
    if step >> 63:
        raise ValueError("step must be below 2^63")
    elem = np.asarray(elem, dtype=np.uint64)
    blk = elem >> np.uint64(4)
    byte = (elem & np.uint64(15)).astype(np.int64)
    ctr = np.stack(
        [
            blk & _U32,
            blk >> np.uint64(32),
            np.full(blk.shape, step & 0xFFFFFFFF, dtype=np.uint64),
            np.full(blk.shape, ((step >> 32) & 0xFFFFFFFF) | 0x80000000, dtype=np.uint64),
        ],
        axis=-1,
    )
    key = np.array([seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF], dtype=np.uint64)
    words = philox4x32_10(ctr, key).astype(np.uint64)
    w = np.take_along_axis(words, (byte >> 2)[..., None], axis=-1)[..., 0]
    b = (w >> (np.uint64(8) * (byte & 3).astype(np.uint64))) & np.uint64(0xFF)
    return b >= np.uint64(threshold)


# --------------------------------------------------------------------------------------------
# Formats (Section 3, "Floating-point formats"): BF16 = 8 exponent / 7 mantissa bits,
# E4M3 = 4 exponent / 3 mantissa bits.
# --------------------------------------------------------------------------------------------


def decode_bf16(bits):
    """BF16 bit patterns (uint16) -> float64, exactly (BF16 is the top half of an FP32)."""
    b = np.asarray(bits).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def _e4m3_value(c):
    """Value of one E4M3 code by the format's definition."""
    s, e, m = (c >> 7) & 1, (c >> 3) & 15, c & 7
    if e == 15 and m == 7:
        return float("nan")
    mag = m * 2.0**-9 if e == 0 else (8 + m) * 2.0 ** (e - 10)
    return -mag if s else mag


_E4M3_VALUES = np.array([_e4m3_value(c) for c in range(256)], dtype=np.float64)


def decode_e4m3(codes):
    """E4M3 codes (uint8) -> float64: (-1)^s 2^(e-7) (1 + m/8); e = 0 is subnormal, 2^-6 m/8;
    e = 15, m = 7 is NaN (OCP flavour, no infinities).  The 256 values are tabulated once."""
    return _E4M3_VALUES[np.asarray(codes).astype(np.uint8)]


def decode(bits, fmt):
    return decode_bf16(bits) if fmt == BF16 else decode_e4m3(bits)


def _split_f32(t):
    t = np.array(t, dtype=np.float32)  # contiguous copy, keeps the shape (also 0-d)
    u = t.view(np.uint32)
    return u >> np.uint32(31), u & np.uint32(0x7FFFFFFF)


def round_bf16(t, r=None):
    """FP32 -> BF16 bits.  r is None: round to nearest, ties to even.  Otherwise r holds the
    16-bit random fields and the result is SR(t) of Eq. (1): the 16 dropped bits plus r carry
    into the kept part with probability (dropped bits) / 2^16 = (t - floor) / (ceil - floor).
    Finite overflow clips to the largest finite BF16; NaN stays NaN."""
    sign, mag = _split_f32(t)
    mag64 = mag.astype(np.uint64)
    if r is None:
        add = np.uint64(0x7FFF) + ((mag64 >> np.uint64(16)) & np.uint64(1))
    else:
        add = np.asarray(r, dtype=np.uint64)
    q = (mag64 + add) >> np.uint64(16)
    q = np.minimum(q, np.uint64(0x7F7F))
    q = np.where(mag > np.uint32(0x7F800000), np.uint64(0x7FC0), q)
    return ((sign.astype(np.uint64) << np.uint64(15)) | q).astype(np.uint16)


def bf16_grid_f64(x):
    """float64 -> nearest BF16 value (ties to even), returned as float64; one rounding straight
    from FP64.  Used for values of modest magnitude (the logit gradient lies in (-1, 1))."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)                       # |x| = f 2^e, f in [0.5, 1)
    ulp = np.exp2(np.maximum(e - 1, -126).astype(np.float64) - 7.0)
    return np.rint(x / ulp) * ulp


def round_e4m3(t, r=None):
    """FP32 -> E4M3 code.  r None: round to nearest even.  Otherwise SR with a 16-bit field.

    The grid F of Eq. (1) is the set of finite E4M3 values.  Below 2^-6 the grid is uniform with
    spacing 2^-9 (subnormals), so |t| 2^9 is rounded as a fixed-point number; from 2^-6 upwards
    each binade has eight steps.  The position of |t| between its grid neighbours is taken to 16
    fractional bits (lower bits dropped) and added to r; a carry rounds away from zero.
    Finite overflow clips to 448; NaN maps to the NaN code."""
    sign, mag = _split_f32(t)
    a = mag.view(np.float32).astype(np.float64)  # |t| exactly
    nan = mag > np.uint32(0x7F800000)
    a = np.where(nan, 0.0, np.minimum(a, 2.0**127))  # infinities clip like any overflow
    sub = a < 2.0**-6
    # exponent of the binade (frexp: a = f 2^e with f in [0.5, 1)) and the grid spacing there
    ex = np.where(sub, -6.0, np.frexp(a)[1].astype(np.float64) - 1.0)
    gap = np.exp2(ex - 3.0)  # 2^-9 in the subnormal range
    pos = a / gap  # exact: power-of-two scaling of an FP32 value
    lo = np.floor(pos)
    frac = pos - lo
    if r is None:
        up = (frac > 0.5) | ((frac == 0.5) & (np.mod(lo, 2.0) == 1.0))
    else:
        f16 = np.floor(frac * 65536.0)
        up = (f16 + np.asarray(r, dtype=np.float64)) >= 65536.0
    val = (lo + up) * gap
    val = np.minimum(val, 448.0)
    # encode the (representable) magnitude
    e2 = np.frexp(val)[1].astype(np.float64) - 1.0
    normal = val >= 2.0**-6
    e_field = np.where(normal, e2 + 7.0, 0.0)
    m_field = np.where(normal, val / np.exp2(e2) * 8.0 - 8.0, val * 512.0)
    code = (e_field * 8 + m_field).astype(np.int64)
    code = np.where(nan, 0x7F, code)
    return ((sign.astype(np.int64) << 7) | code).astype(np.uint8)


def round_em(t, exp_bits, man_bits, r=None):
    """FP32 -> the nearest (r None, ties to even) or stochastically rounded (16-bit field r)
    value of a simulated floating-point format with `exp_bits` exponent and `man_bits` mantissa
    bits, returned as FP32 -- the tool of the bit-width study of Section 4.3 ("simulating
    floating-point numbers with a specific number of mantissa and exponent bits").

    Reading (the paper gives no definition): the IEEE-754 pattern -- bias 2^(E-1)-1, the top
    exponent code reserved, gradual underflow -- so that (8,7) is BF16, (5,10) FP16 and (5,2)
    E5M2; finite overflow and infinities clip to the largest finite value, NaN stays NaN, the
    sign of a zero result is kept.  SR as everywhere here: the position of |t| between its two
    grid neighbours, cut to 16 fractional bits, plus r carries or not (Eq. 1 with probabilities
    in steps of 2^-16)."""
    E, M = int(exp_bits), int(man_bits)
    assert 2 <= E <= 8 and 1 <= M <= 22
    sign, mag = _split_f32(t)
    a = mag.view(np.float32).astype(np.float64)
    nan = mag > np.uint32(0x7F800000)
    a = np.where(nan, 0.0, a)
    emax, emin = 2 ** (E - 1) - 1, 2 - 2 ** (E - 1)
    top = (2.0 - 2.0 ** -M) * 2.0 ** emax
    a = np.minimum(a, 2.0 * top)                     # infinities clip like any overflow
    ex = np.maximum(np.frexp(a)[1].astype(np.float64) - 1.0, float(emin))
    gap = np.exp2(ex - M)                            # grid spacing in the binade of |t| (subnormal: 2^(emin-M))
    pos = a / gap
    lo = np.floor(pos)
    frac = pos - lo
    if r is None:
        up = (frac > 0.5) | ((frac == 0.5) & (np.mod(lo, 2.0) == 1.0))
    else:
        up = (np.floor(frac * 65536.0) + np.asarray(r, dtype=np.float64)) >= 65536.0
    val = np.minimum((lo + up) * gap, top)
    out = np.where(sign.astype(bool), -val, val).astype(np.float32)
    return np.where(nan, np.asarray(t, dtype=np.float32), out)


def quantize(t, fmt, r=None):
    return round_bf16(t, r) if fmt == BF16 else round_e4m3(t, r)


# --------------------------------------------------------------------------------------------
# The head step (Algorithm 1; gradients from the appendix on skipping the loss)
# --------------------------------------------------------------------------------------------


def csr_to_dense(indptr, indices, n_cols, col_ids=None):
    """Dense 0/1 matrix Y[B, n] of the positives.  col_ids (ascending global label ids) selects
    the columns; None means all n_cols labels."""
    B = len(indptr) - 1
    if col_ids is None:
        Y = np.zeros((B, n_cols), dtype=np.float64)
        for i in range(B):
            Y[i, indices[indptr[i]:indptr[i + 1]]] = 1.0
        return Y
    col_ids = np.asarray(col_ids, dtype=np.int64)
    Y = np.zeros((B, len(col_ids)), dtype=np.float64)
    for i in range(B):
        row = np.asarray(indices[indptr[i]:indptr[i + 1]], dtype=np.int64)
        pos = np.searchsorted(col_ids, row)
        ok = (pos < len(col_ids))
        ok[ok] &= col_ids[pos[ok]] == row[ok]
        Y[i, pos[ok]] = 1.0
    return Y


def sigmoid(z):
    """1 / (1 + e^-z), evaluated without overflow for large |z|."""
    z = np.asarray(z, dtype=np.float64)
    ez = np.exp(-np.abs(z))
    return np.where(z >= 0, 1.0 / (1.0 + ez), ez / (1.0 + ez))


def logits_inputs(X_bits, fmt):
    """Decoded inputs of the logits product: in E4M3 mode the BF16 inputs are first cast to E4M3
    (round to nearest even), in BF16 mode they are used as they are (Algorithm 1; Section 4.1)."""
    X = decode_bf16(X_bits)
    if fmt == E4M3:
        return decode_e4m3(round_e4m3(X.astype(np.float32)))
    return X


def logits(W_bits, X_bits, fmt):
    """Z[B, n] = Xq W^T in FP64 for the given weight rows."""
    return logits_inputs(X_bits, fmt) @ decode(W_bits, fmt).T


def logit_gradient(Z, Y, g_exact=False):
    """G = sigmoid(Z) - Y, the 'classifier logit gradient', held in BF16 (Section 4.4): one
    round-to-nearest-even of the FP64 value.  g_exact=True returns the unrounded FP64 values."""
    G = sigmoid(Z) - Y
    return G if g_exact else bf16_grid_f64(G)


def bce_loss(Z, Y):
    """Sum over all (sample, label) of softplus(z) - y z, whose derivative w.r.t. Z is G."""
    return float(np.sum(np.maximum(Z, 0.0) + np.log1p(np.exp(-np.abs(Z))) - Y * Z))


def update_rows(W_bits, comp_bits, dW, lr, fmt, flags, seed, step, elem, weight_decay=0.0):
    """Fused SGD update of weight elements (Algorithm 1, fuse_update; Section 3 Kahan).

    W_bits/comp_bits/dW/elem have the same shape; elem holds the flat element indices that pick
    the random fields.  FP32 arithmetic, each operation rounded once:
        g = fl(dW); u = fl(lr g)
      plain : t = fl(w - u);                      w' = Q(t)
      Kahan : y = fl(-u - c); t = fl(w + y);      w' = Q(t);  c' = RNE_BF16(fl(fl(w' - w) - y))
    Q is SR (flag SR) or round-to-nearest-even.  Returns (W_bits', comp_bits' or None).

    weight_decay (the classifier's "WD" of the hyper-parameter table; Algorithm 1 leaves it out,
    reading: the L2 term of plain SGD added to the gradient): g = fl(g + fl(wd w)) before the
    steps above; 0 skips the two operations.
    """
    f32 = np.float32
    w = decode(W_bits, fmt).astype(f32)  # exact
    g = np.asarray(dW, dtype=np.float64).astype(f32)
    if weight_decay != 0.0:
        g = (g + (f32(weight_decay) * w).astype(f32)).astype(f32)
    u = (f32(lr) * g).astype(f32)
    r = sr_fields(seed, step, elem) if (flags & FLAG_SR) else None
    if flags & FLAG_KAHAN:
        c = decode_bf16(comp_bits).astype(f32)
        y = ((-u) - c).astype(f32)
        t = (w + y).astype(f32)
        Wn = quantize(t, fmt, r)
        wn = decode(Wn, fmt).astype(f32)
        with np.errstate(invalid="ignore"):
            cn = ((wn - w).astype(f32) - y).astype(f32)
        return Wn, round_bf16(cn)
    t = (w - u).astype(f32)
    return quantize(t, fmt, r), None


def head_step(W_bits, comp_bits, X_bits, indptr, indices, lr, seed, step, fmt, flags,
              label_ids=None, g_exact=False, kahan_rows=None, weight_decay=0.0, dropout=0):
    """One training step of the head on the given weight rows.

    dropout (threshold T in [0, 255], 0 = none; appendix "Low-Memory Dropout for Classifier"):
    this step's weights are W o M / (1 - T/256) with the keep mask M of dropout_keep.  Reading: the
    same masked weights serve the logits and the input gradient, and the weight gradient is that
    of the masked model (zero where M is zero, scaled elsewhere) -- what differentiating the loss
    of the masked model gives; the update itself (decay, Kahan, rounding) acts on the stored W.

    kahan_rows (with FLAG_KAHAN; None = every label): only the labels with id < kahan_rows carry a
    compensation value -- the paper's "Kahan summation for head labels" (appendix "Precision
    Recovery for Sensitive Applications"), with the labels numbered by falling frequency so that
    the top-p% head is a prefix.  The other labels are updated as without the flag; their rows of
    comp_bits are ignored and come back unchanged.

    W_bits [n, d] (uint16 BF16 patterns or uint8 E4M3 codes), comp_bits [n, d] uint16 or None,
    X_bits [B, d] uint16 (BF16), CSR positives over global label ids.  label_ids gives the global
    label id of each row of W_bits (None: rows are labels 0..n-1); it selects the positives and
    the random fields, so a subset of rows gives exactly the rows of the full result.

    Returns dict with Z, G (FP64, [B, n]), dX_partial = G W_old (FP64, [B, d]; the full input
    gradient when all labels are given), dW = G^T X (FP64), W_new, comp_new, loss.
    """
    W_bits = np.asarray(W_bits)
    n, d = W_bits.shape
    if label_ids is None:
        label_ids = np.arange(n, dtype=np.int64)
    label_ids = np.asarray(label_ids, dtype=np.int64)
    Wd = decode(W_bits, fmt)
    elem = label_ids[:, None] * np.int64(d) + np.arange(d, dtype=np.int64)[None, :]
    if dropout:
        keep = dropout_keep(seed, step, elem, dropout)
        scale = 256.0 / (256.0 - dropout)
        Wd = np.where(keep, Wd, 0.0) * scale        # the weights this step's products see
    X = decode_bf16(X_bits)
    Xq = logits_inputs(X_bits, fmt)
    Z = Xq @ Wd.T
    Y = csr_to_dense(indptr, indices, None, col_ids=label_ids)
    G = logit_gradient(Z, Y, g_exact)
    dX = G @ Wd            # weights before the update (the update comes later in Algorithm 1)
    dW = G.T @ X           # BF16 inputs, summed over the batch, no 1/B
    if dropout:
        dW = np.where(keep, dW, 0.0) * scale
    if (flags & FLAG_KAHAN) and kahan_rows is not None:
        head = label_ids < kahan_rows
        comp_bits = np.asarray(comp_bits)
        Wn, cn = np.array(W_bits, copy=True), np.array(comp_bits, copy=True)
        if head.any():
            Wn[head], cn[head] = update_rows(W_bits[head], comp_bits[head], dW[head], lr, fmt, flags, seed, step, elem[head], weight_decay)
        if (~head).any():
            Wn[~head], _ = update_rows(W_bits[~head], None, dW[~head], lr, fmt, flags & ~FLAG_KAHAN, seed, step, elem[~head], weight_decay)
    else:
        Wn, cn = update_rows(W_bits, comp_bits, dW, lr, fmt, flags, seed, step, elem, weight_decay)
    return dict(Z=Z, G=G, dX_partial=dX, dW=dW, W_new=Wn, comp_new=cn, loss=bce_loss(Z, Y))


def input_gradient_rows(W_bits, X_bits, indptr, indices, fmt, rows, block=65536, g_exact=False,
                        dropout=0, seed=0, step=0):
    """Rows `rows` of the full input gradient dX = (sigmoid(Xq W^T) - Y) W over all labels,
    streaming the weight rows in blocks so that millions of labels fit in memory.  Also returns
    the logits of those rows, Z[len(rows), L]."""
    rows = np.asarray(rows, dtype=np.int64)
    L, d = W_bits.shape
    Xq = logits_inputs(np.asarray(X_bits)[rows], fmt)
    sub_ptr = [0]
    sub_idx = []
    for i in rows:
        sub_idx.append(np.asarray(indices[indptr[i]:indptr[i + 1]], dtype=np.int64))
        sub_ptr.append(sub_ptr[-1] + len(sub_idx[-1]))
    sub_idx = np.concatenate(sub_idx) if sub_idx else np.zeros(0, np.int64)
    dX = np.zeros((len(rows), d), dtype=np.float64)
    Z = np.empty((len(rows), L), dtype=np.float64)
    for l0 in range(0, L, block):
        l1 = min(L, l0 + block)
        Wd = decode(W_bits[l0:l1], fmt)
        if dropout:
            elem = np.arange(l0, l1, dtype=np.int64)[:, None] * np.int64(d) + np.arange(d, dtype=np.int64)[None, :]
            Wd = np.where(dropout_keep(seed, step, elem, dropout), Wd, 0.0) * (256.0 / (256.0 - dropout))
        z = Xq @ Wd.T
        Y = csr_to_dense(sub_ptr, sub_idx, None, col_ids=np.arange(l0, l1))
        dX += logit_gradient(z, Y, g_exact) @ Wd
        Z[:, l0:l1] = z
    return dX, Z


def topk(Z, k):
    """Indices and scores of the k largest entries of each row of Z, ordered by (score
    descending, label id ascending) -- the top_k of the P@k definition."""
    Z = np.asarray(Z, dtype=np.float64)
    ids = np.arange(Z.shape[1])
    idx = np.empty((Z.shape[0], k), dtype=np.int64)
    for i in range(Z.shape[0]):
        order = np.lexsort((ids, -Z[i]))
        idx[i] = order[:k]
    return idx, np.take_along_axis(Z, idx, axis=1)


def precision_hits(idx, indptr, indices):
    """Numerators of P@k (evaluation section, "Precision at k"): hits[j-1] = number of (row, label)
    pairs with the label among the row's first j predictions and among its true labels, summed
    over the rows, for j = 1..k.  P@j = hits[j-1] / (j * rows).  idx [rows, k], best first."""
    idx = np.asarray(idx)
    rows, k = idx.shape
    hits = np.zeros(k, dtype=np.int64)
    for i in range(rows):
        truth = set(int(l) for l in indices[indptr[i]:indptr[i + 1]])
        for j in range(k):
            if int(idx[i, j]) in truth:
                hits[j:] += 1
    return hits


def kahan_sum_stream(s_bits, c_bits, addends, fmt):
    """Apply the Kahan recurrence of Section 3 repeatedly to one stored value: s in `fmt`,
    c in BF16, each v of `addends` added with FP32 arithmetic and round-to-nearest storage.
    Returns the final (s_bits, c_bits).  Used by the tests of the recurrence."""
    f32 = np.float32
    s_bits = np.asarray(s_bits)
    c_bits = np.asarray(c_bits)
    for v in addends:
        s = decode(s_bits, fmt).astype(f32)
        c = decode_bf16(c_bits).astype(f32)
        y = (f32(v) - c).astype(f32)
        t = (s + y).astype(f32)
        s_new_bits = quantize(t, fmt)
        s_new = decode(s_new_bits, fmt).astype(f32)
        c_bits = round_bf16(((s_new - s).astype(f32) - y).astype(f32))
        s_bits = s_new_bits
    return s_bits, c_bits


def kahan_adamw(p_bits, c_bits, m, v, g_bits, lr, beta1, beta2, eps, weight_decay, t, wide=False):
    """One AdamW step with Kahan-compensated BF16 parameters -- what Section 4.1 uses for the
    encoder ("Kahan summation for the encoder's parameters"; the experimental set-up names a fused
    Kahan-AdamW).  AdamW is Loshchilov & Hutter's: decoupled weight decay, bias-corrected moments.

    p_bits, c_bits, g_bits: uint16 BF16 patterns (parameter, compensation, gradient).  m, v: the
    moments, uint16 BF16 patterns or float32 arrays (kept in the type they arrive in).  t >= 1 is
    the step count of the bias correction.  Reading (the paper defers to a library): FP32
    arithmetic, every operation rounded once, in this order
        m' = fl(fl(b1 m) + fl(o1 g));              v' = fl(fl(b2 v) + fl(fl(o2 g) g))
        mh = fl(m' / bc1);  vh = fl(v' / bc2)
    with the scalars b_i = fl32(beta_i), o_i = fl32(1 - beta_i), bc_i = fl32(1 - beta_i^t) formed in
    FP64 from the FP64 betas and rounded once,
    then
        r  = fl(mh / fl(fl(sqrt(vh)) + eps));      r = fl(r + fl(wd p)) if wd != 0
        u  = fl(lr r)
        y  = fl(-u - c);  s = fl(p + y);  p' = RNE_BF16(s);  c' = RNE_BF16(fl(fl(p' - p) - y))
    (the last line is the Kahan recurrence of Section 3 with the update -u as the addend), and the
    moments are stored round-to-nearest-even when they are BF16.

    wide=True is the same recipe in FP64 with nothing rounded and p, c, m, v, g given as float64
    values (c is then always 0): the textbook AdamW the tests compare with torch's.
    Returns (p, c, m, v) in the types they came in.
    """
    if wide:
        p, c, m, v, g = (np.asarray(a, dtype=np.float64) for a in (p_bits, c_bits, m, v, g_bits))
        m1 = beta1 * m + (1.0 - beta1) * g
        v1 = beta2 * v + (1.0 - beta2) * g * g
        r = (m1 / (1.0 - beta1 ** t)) / (np.sqrt(v1 / (1.0 - beta2 ** t)) + eps)
        r = r + weight_decay * p
        return p - lr * r - c, np.zeros_like(p), m1, v1
    f32 = np.float32
    p = decode_bf16(p_bits).astype(f32)
    c = decode_bf16(c_bits).astype(f32)
    g = decode_bf16(g_bits).astype(f32)
    m_is_bf16 = np.asarray(m).dtype == np.uint16
    v_is_bf16 = np.asarray(v).dtype == np.uint16
    m0 = decode_bf16(m).astype(f32) if m_is_bf16 else np.asarray(m, dtype=f32)
    v0 = decode_bf16(v).astype(f32) if v_is_bf16 else np.asarray(v, dtype=f32)
    b1, b2 = f32(beta1), f32(beta2)
    ob1, ob2 = f32(1.0 - beta1), f32(1.0 - beta2)
    bc1, bc2 = f32(1.0 - beta1 ** t), f32(1.0 - beta2 ** t)
    m1 = ((b1 * m0).astype(f32) + (ob1 * g).astype(f32)).astype(f32)
    v1 = ((b2 * v0).astype(f32) + ((ob2 * g).astype(f32) * g).astype(f32)).astype(f32)
    mh = (m1 / bc1).astype(f32)
    vh = (v1 / bc2).astype(f32)
    r = (mh / (np.sqrt(vh).astype(f32) + f32(eps)).astype(f32)).astype(f32)
    if weight_decay != 0.0:
        r = (r + (f32(weight_decay) * p).astype(f32)).astype(f32)
    u = (f32(lr) * r).astype(f32)
    y = ((-u) - c).astype(f32)
    s_ = (p + y).astype(f32)
    p_new_bits = round_bf16(s_)
    p_new = decode_bf16(p_new_bits).astype(f32)
    c_new_bits = round_bf16(((p_new - p).astype(f32) - y).astype(f32))
    m_out = round_bf16(m1) if m_is_bf16 else m1
    v_out = round_bf16(v1) if v_is_bf16 else v1
    return p_new_bits, c_new_bits, m_out, v_out
