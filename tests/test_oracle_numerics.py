"""Pins of the oracle's number formats, random fields, stochastic rounding and Kahan recurrence
against things other than the oracle itself: the published Philox vectors, torch's CPU casts,
exhaustive enumeration of the 16-bit random field, closed forms."""
import os

import numpy as np
import pytest
import torch

from oracle import elmo_oracle as o

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- Philox
def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(x, 16) for x in line.split()])
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for r in rows:
        out = o.philox4x32_10(r[0:4], r[4:6])
        assert [int(x) for x in out] == r[6:10]


def test_philox_vectorised_matches_scalar_calls():
    rng = np.random.default_rng(5)
    ctr = rng.integers(0, 2**32, size=(17, 4), dtype=np.uint64)
    key = rng.integers(0, 2**32, size=(2,), dtype=np.uint64)
    batch = o.philox4x32_10(ctr, key)
    for i in range(17):
        assert np.array_equal(batch[i], o.philox4x32_10(ctr[i], key))


def test_sr_field_layout():
    """Element e takes 16-bit field e % 8 of block e // 8; counter = (block, step), key = seed."""
    seed = 0x0123456789ABCDEF
    step = 0x1122334455667788
    e = np.array([0, 1, 2, 7, 8, 15, 8 * (2**33 + 5) + 3], dtype=np.uint64)
    got = o.sr_fields(seed, step, e)
    for ei, gi in zip(e.tolist(), got.tolist()):
        blk, f = divmod(ei, 8)
        words = o.philox4x32_10(
            [blk & 0xFFFFFFFF, blk >> 32, step & 0xFFFFFFFF, step >> 32],
            [seed & 0xFFFFFFFF, seed >> 32])
        w = int(words[f // 2])
        assert gi == (w >> (16 * (f % 2))) & 0xFFFF


def test_sr_fields_change_with_seed_and_step_and_look_uniform():
    e = np.arange(1 << 20, dtype=np.uint64)
    a = o.sr_fields(0, 0, e)
    assert not np.array_equal(a, o.sr_fields(0, 1, e))
    assert not np.array_equal(a, o.sr_fields(1, 0, e))
    assert np.array_equal(a, o.sr_fields(0, 0, e))
    hist = np.bincount(a >> 8, minlength=256).astype(np.float64)   # 256 cells, df = 255
    chi2 = np.sum((hist - len(e) / 256) ** 2 / (len(e) / 256))
    assert 160 < chi2 < 370          # roughly +-4.5 sigma around 255
    assert abs(a.mean() - 32767.5) < 5 * 65536 / np.sqrt(12 * len(e))


# ----------------------------------------------------------------------------- formats
def test_e4m3_decode_closed_form_and_torch():
    codes = np.arange(256, dtype=np.uint8)
    got = o.decode_e4m3(codes)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.array_equal(got[~np.isnan(got)], ref[~np.isnan(ref)])
    # hand values: the paper quotes the exponent range [-9, 8]: smallest 2^-9, largest 1.75 * 2^8
    assert got[0x01] == 2.0**-9 and got[0x7E] == 448.0 and got[0x08] == 2.0**-6
    assert got[0x38] == 1.0 and got[0xB8] == -1.0 and np.isnan(got[0x7F]) and np.isnan(got[0xFF])
    assert np.signbit(got[0x80]) and got[0x80] == 0.0


def test_bf16_decode_is_top_half_of_fp32():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = o.decode_bf16(bits)
    ok = ~np.isnan(ref)
    assert np.array_equal(np.isnan(got), ~ok) and np.array_equal(got[ok], ref[ok])


def _spread_f32(n, lo, hi, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(n) * np.exp(rng.uniform(lo, hi, n))).astype(np.float32)


def test_rne_bf16_matches_torch_cast():
    x = np.concatenate([_spread_f32(1 << 21, -85, 85, 1),
                        np.array([0.0, -0.0, 1e-40, -1e-45, 3.3e38], dtype=np.float32)])
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    finite = np.isfinite(torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())
    got = o.round_bf16(x)
    assert np.array_equal(got[finite], ref[finite])
    # every mantissa pattern of one binade, including all ties
    u = (np.uint32(0x3F800000) + np.arange(1 << 23, dtype=np.uint32)).view(np.float32)
    ref = torch.from_numpy(u).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(o.round_bf16(u), ref)


def test_rne_bf16_hand_cases():
    f = np.float32
    # spacing at 1 is 2^-7: 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> 1 + 2^-6
    cases = {1.0 + 2.0**-8: 0x3F80, 1.0 + 3 * 2.0**-8: 0x3F82, 1.0 + 2.0**-8 + 2.0**-20: 0x3F81,
             -(1.0 + 2.0**-8): 0xBF80}
    for x, want in cases.items():
        assert int(o.round_bf16(f(x))) == want
    # finite overflow clips to the largest finite value (reading: clipping error), NaN stays NaN
    assert int(o.round_bf16(f(3.4e38))) == 0x7F7F
    assert int(o.round_bf16(f(-np.inf))) == 0xFF7F
    assert (int(o.round_bf16(f(np.nan))) & 0x7FFF) == 0x7FC0


def test_rne_e4m3_matches_torch_cast_where_torch_is_finite():
    x = np.concatenate([_spread_f32(1 << 21, -14, 6.2, 2),
                        np.array([0.0, -0.0, 2.0**-10, 3 * 2.0**-10, 2.0**-6, 448, 464, -464, 1e-30],
                                 dtype=np.float32)])
    x = x[np.abs(x) <= 464]
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(o.round_e4m3(x), ref)


def test_rne_e4m3_roundtrip_ties_and_clipping():
    codes = np.arange(256, dtype=np.uint8)
    finite = (codes & 0x7F) != 0x7F
    v = o.decode_e4m3(codes[finite]).astype(np.float32)
    assert np.array_equal(o.round_e4m3(v), codes[finite])
    f = np.float32
    assert int(o.round_e4m3(f(2.0**-10))) == 0x00          # tie between 0 and 2^-9 -> even (0)
    assert int(o.round_e4m3(f(3 * 2.0**-10))) == 0x02      # tie between 1 and 2 steps -> 2
    assert int(o.round_e4m3(f(1.0625))) == 0x38            # tie 1.0 / 1.125 -> even mantissa
    assert int(o.round_e4m3(f(1.1875))) == 0x3A            # tie 1.125 / 1.25 -> 1.25
    assert int(o.round_e4m3(f(-0.0))) == 0x80
    assert int(o.round_e4m3(f(-1e-9))) == 0x80             # rounds to zero, keeps its sign
    assert int(o.round_e4m3(f(1e9))) == 0x7E and int(o.round_e4m3(f(-np.inf))) == 0xFE
    assert int(o.round_e4m3(f(465.0))) == 0x7E             # clips (torch's cast gives NaN here)
    assert (int(o.round_e4m3(f(np.nan))) & 0x7F) == 0x7F
    # upper end of the subnormal range rounds up into the first normal code
    assert int(o.round_e4m3(f(2.0**-6 - 2.0**-12))) == 0x08


def test_bf16_grid_rounds_once_from_fp64():
    """The BF16 rounding of the FP64 logit gradient: equals the FP32 route wherever FP32 holds the
    value exactly, and does not double-round where it does not."""
    x32 = _spread_f32(1 << 18, -30, 1, 7)
    np.testing.assert_array_equal(o.bf16_grid_f64(x32.astype(np.float64)), o.decode_bf16(o.round_bf16(x32)))
    assert o.bf16_grid_f64(1.0 + 2.0**-8) == 1.0                       # tie -> even
    assert o.bf16_grid_f64(1.0 + 2.0**-8 + 2.0**-40) == 1.0 + 2.0**-7  # just above the tie
    assert o.bf16_grid_f64(-0.3) == -0.30078125 and o.bf16_grid_f64(0.0) == 0.0
    from fractions import Fraction
    rng = np.random.default_rng(0)
    for x in rng.uniform(-1, 1, 200):
        e = np.frexp(x)[1] - 1
        ulp = Fraction(2) ** int(e - 7)
        q = Fraction(float(x)) / ulp
        lo = q.numerator // q.denominator
        r = q - lo
        n = lo + (1 if (r > Fraction(1, 2) or (r == Fraction(1, 2) and lo % 2 == 1)) else 0)
        assert Fraction(float(o.bf16_grid_f64(x))) == n * ulp


# ----------------------------------------------------------------------------- SR, Eq. (1)
def _grid(fmt):
    if fmt == o.E4M3:
        c = np.arange(0x7F, dtype=np.uint8)
        return np.sort(o.decode_e4m3(c))
    raise ValueError


def _neighbours_e4m3(a):
    g = _grid(o.E4M3)
    hi = g[np.searchsorted(g, a, side="left")]
    lo = g[np.searchsorted(g, a, side="right") - 1]
    return lo, hi


ALL_R = np.arange(65536, dtype=np.uint32)


@pytest.mark.parametrize("t", [0.3, -0.3, 0.0123, 1.0 + 2.0**-10, 300.1, 2.0**-6 + 2.0**-13,
                               2.0**-9 * 0.37, -(2.0**-9) * 5.62, 440.0, 1e-5])
def test_sr_e4m3_enumeration_over_all_fields(t):
    t = np.float32(t)
    a = abs(float(t))
    lo, hi = _neighbours_e4m3(a)
    out = o.decode_e4m3(o.round_e4m3(np.full(65536, t, np.float32), ALL_R))
    mags = np.abs(out)
    assert set(np.unique(mags).tolist()) <= {lo, hi}             # only the two neighbours
    assert np.all(np.signbit(out) == np.signbit(t))
    p = (a - lo) / (hi - lo)
    ups = int(np.sum(mags == hi))
    assert ups == int(np.floor(p * 65536))                       # Eq. (1), to 16 bits, rounded down
    # increasing r can only turn a round-down into a round-up
    assert np.all(np.diff((mags == hi).astype(np.int8)) >= 0)


@pytest.mark.parametrize("t", [0.3, -0.02, 1.0 + 2.0**-9, 3.0e38, 1e-39, -7.77e-12, 123456.7])
def test_sr_bf16_enumeration_is_eq1_exactly(t):
    t = np.float32(t)
    bits = o.round_bf16(np.full(65536, t, np.float32), ALL_R)
    out = o.decode_bf16(bits)
    lo_bits = np.uint16(np.float32(t).view(np.uint32) >> 16)
    lo = float(o.decode_bf16(lo_bits))
    hi = float(o.decode_bf16(np.uint16(lo_bits + 1)))
    assert set(np.unique(out).tolist()) <= {lo, hi}
    p = (float(t) - lo) / (hi - lo)                               # exact in FP64
    assert int(np.sum(out == hi)) == int(round(p * 65536)) and p * 65536 == round(p * 65536)


def test_sr_leaves_representable_values_alone_and_clips():
    codes = np.arange(256, dtype=np.uint8)
    codes = codes[(codes & 0x7F) != 0x7F]
    v = o.decode_e4m3(codes).astype(np.float32)
    for r in (0, 1, 0x8000, 0xFFFF):
        assert np.array_equal(o.round_e4m3(v, np.full(v.shape, r, np.uint32)), codes)
    b = np.array([0x0000, 0x8000, 0x3F80, 0x0001, 0x7F7F, 0xC2F7], dtype=np.uint16)
    vb = o.decode_bf16(b).astype(np.float32)
    for r in (0, 0xFFFF):
        assert np.array_equal(o.round_bf16(vb, np.full(vb.shape, r, np.uint32)), b)
    # beyond the largest finite value every draw clips to it
    assert set(o.round_e4m3(np.full(65536, 460.0, np.float32), ALL_R).tolist()) == {0x7E}
    assert set(o.round_bf16(np.full(65536, 3.4e38, np.float32), ALL_R).tolist()) == {0x7F7F}


@pytest.mark.parametrize("fmt,x", [(o.E4M3, 0.3), (o.E4M3, -0.0123), (o.E4M3, 2.0**-9 * 2.3),
                                   (o.E4M3, 437.0), (o.BF16, 0.7123456), (o.BF16, -1.00001e-3),
                                   (o.BF16, 5.4321e20)])
def test_sr_mean_over_1e6_philox_draws_within_3_sigma(fmt, x):
    x = np.float32(x)
    n = 1_000_000
    r = o.sr_fields(12345, 7, np.arange(n, dtype=np.uint64))
    out = o.decode(o.quantize(np.full(n, x, np.float32), fmt, r), fmt)
    vals = np.unique(out)
    assert len(vals) == 2
    gap = vals[1] - vals[0]
    p = (float(x) - vals[0]) / gap
    sigma = gap * np.sqrt(p * (1 - p) / n)
    assert abs(out.mean() - float(x)) < 3 * sigma


# ----------------------------------------------------------------------------- Kahan
def test_kahan_special_case_exact_sum_has_zero_compensation():
    s = o.round_bf16(np.float32(1.0))
    s2, c2 = o.kahan_sum_stream(s, np.uint16(0), [0.5], o.BF16)
    assert float(o.decode_bf16(s2).item()) == 1.5 and float(o.decode_bf16(c2).item()) == 0.0


def test_small_updates_cancel_under_rne_but_kahan_tracks_them():
    """Section 4.1: an update below half the spacing is cancelled by round-to-nearest.  With the
    compensation term of Section 3 the stored pair (s, c) follows the true sum."""
    for fmt, s0, v, n in [(o.BF16, 1.0, 2.0**-10, 10_000), (o.E4M3, 0.25, 2.0**-8, 100)]:
        s_bits = o.quantize(np.float32(s0), fmt)
        # plain round-to-nearest accumulation: bit-identical after 10^4 updates
        sb = s_bits
        for _ in range(50):
            sb = o.quantize((o.decode(sb, fmt).astype(np.float32) + np.float32(v)).astype(np.float32), fmt)
        assert sb == s_bits
        sk, ck = o.kahan_sum_stream(s_bits, np.uint16(0), [v] * n, fmt)
        true = s0 + n * v
        sv = float(np.asarray(o.decode(sk, fmt)).item())
        est = sv - float(np.asarray(o.decode_bf16(ck)).item())
        ulp = {o.BF16: 2.0**-7, o.E4M3: 2.0**-3}[fmt] * 2 ** np.floor(np.log2(true))
        assert abs(sv - true) <= ulp            # s itself within one spacing
        assert abs(est - true) <= ulp * 2.0**-6                        # s - c far closer


def test_kahan_random_walk_error_stays_bounded():
    rng = np.random.default_rng(3)
    v = (rng.standard_normal(4000) * 1e-3).astype(np.float32)
    s_bits, c_bits = o.kahan_sum_stream(o.round_bf16(np.float32(0.5)), np.uint16(0), v, o.BF16)
    true = 0.5 + np.sum(v.astype(np.float64))
    s = float(np.asarray(o.decode_bf16(s_bits)).item())
    c = float(np.asarray(o.decode_bf16(c_bits)).item())
    ulp_s = 2.0**-7 * 2 ** np.floor(np.log2(abs(true)))
    assert abs(s - true) <= ulp_s
    # c is itself stored in BF16: each step loses at most half a spacing of c (|c| <= ulp_s / 2)
    assert abs((s - c) - true) <= 4000 * (ulp_s / 2) * 2.0**-8
    # without compensation the same stream drifts by many spacings or stalls
    sb = o.round_bf16(np.float32(0.5))
    for x in v:
        sb = o.round_bf16((o.decode_bf16(sb).astype(np.float32) + x).astype(np.float32))
    assert abs(float(np.asarray(o.decode_bf16(sb)).item()) - true) > abs(s - c - true)


# --------------------------------------------------------------------------------------------
# Simulated (exponent, mantissa) formats (Section 4.3): pinned to torch's casts of the three
# IEEE-pattern formats it has, and to this module's own BF16 / E4M3 rules where they coincide
# --------------------------------------------------------------------------------------------
def _em_inputs(limit):
    rng = np.random.default_rng(77)
    x = np.concatenate([
        (rng.standard_normal(20000) * 10.0 ** rng.uniform(-9, 4, 20000)).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 0.1, 1.5, 2.0 ** -14, 2.0 ** -15, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25,
                  65504.0, 57344.0, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.25, 1.375, 1.125], dtype=np.float32)])
    return x[np.abs(x) <= limit]


@pytest.mark.parametrize("E,M,dtype,limit", [
    (8, 7, torch.bfloat16, 3.0e38),
    (5, 10, torch.float16, 65504.0),
    (5, 2, torch.float8_e5m2, 57344.0),
])
def test_simulated_format_equals_torch_cast(E, M, dtype, limit):
    x = _em_inputs(limit)
    want = torch.from_numpy(x).to(dtype).to(torch.float32).numpy()
    got = o.round_em(x, E, M)
    np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))


def test_simulated_format_special_values_and_sr():
    # overflow clips (no infinities), NaN stays, sign of zero kept
    big = np.array([1e30, -1e30, np.inf, -np.inf], np.float32)
    np.testing.assert_array_equal(o.round_em(big, 5, 2), np.array([57344, -57344, 57344, -57344], np.float32))
    assert np.isnan(o.round_em(np.array([np.nan], np.float32), 4, 3)[0])
    assert np.signbit(o.round_em(np.array([-1e-30], np.float32), 5, 10)[0])
    # (8,7) with a field is this module's BF16 stochastic rounding, (4,3) its E4M3 one below the
    # IEEE-pattern limit 240 (E4M3 of Algorithm 1 is the non-IEEE "FN" flavour that goes on to 448)
    x = _em_inputs(200.0)
    r = np.random.default_rng(5).integers(0, 65536, x.shape)
    np.testing.assert_array_equal(o.round_em(x, 8, 7, r), o.decode_bf16(o.round_bf16(x, r)).astype(np.float32))
    np.testing.assert_array_equal(o.round_em(x, 4, 3, r), o.decode_e4m3(o.round_e4m3(x, r)).astype(np.float32))
    np.testing.assert_array_equal(o.round_em(x, 4, 3), o.decode_e4m3(o.round_e4m3(x)).astype(np.float32))
    # Eq. (1) by enumeration for a 3-bit mantissa: x = 1 + 3/32 lies 3/4 of the way from 1 to 1.125
    ups = sum(float(o.round_em(np.float32(1.09375), 3, 3, np.array(rr))) == 1.125 for rr in range(0, 65536, 64))
    assert ups == 1024 * 3 // 4


def _em_grid(E, M):
    """Every non-negative value of the (E, M) format of the IEEE pattern, as exact fractions, in
    ascending order, with the mantissa code's parity (for ties to even)."""
    from fractions import Fraction
    bias = 2 ** (E - 1) - 1
    vals = []
    for e in range(0, 2 ** E - 1):                   # the top exponent code is reserved
        for m in range(2 ** M):
            v = Fraction(m, 2 ** M) * Fraction(2) ** (1 - bias) if e == 0 else (1 + Fraction(m, 2 ** M)) * Fraction(2) ** (e - bias)
            vals.append((v, (e * 2 ** M + m) & 1))
    return vals


@pytest.mark.parametrize("E,M", [(3, 4), (2, 1), (4, 3), (6, 9)])
def test_simulated_format_against_a_brute_force_over_its_whole_grid(E, M):
    """Formats torch has no cast for: the oracle's formula against the definition carried out in
    exact rational arithmetic -- enumerate every value of the format, find the two neighbours of
    |x| by search, round to the nearer one (ties to the even code) or, stochastically, up iff
    floor(2^16 (|x| - lo) / (hi - lo)) + r >= 2^16 -- on inputs in the subnormal range of the
    format, across the subnormal / normal boundary, on grid points and midpoints, next to the
    largest finite value and beyond it."""
    import bisect
    from fractions import Fraction
    grid = _em_grid(E, M)
    gv = [v for v, _ in grid]
    top = gv[-1]
    rng = np.random.default_rng(E * 100 + M)
    pts = [float(v) for v in rng.choice(np.array([float(x) for x in gv]), 60)]
    mids = [float((gv[i] + gv[i + 1]) / 2) for i in rng.integers(0, len(gv) - 1, 60)] + [float((gv[0] + gv[1]) / 2), float((gv[-2] + gv[-1]) / 2)]
    sub = (rng.random(80) * float(gv[2 ** M]) * 1.5).tolist()                  # subnormals and the first normals
    near_top = (float(top) * (1 + rng.uniform(-2.0 ** -M, 2.0 ** -M, 40))).tolist() + [float(top) * 1.5, float(top) * 64, 3.0e38]
    wide = (np.exp(rng.uniform(np.log(float(gv[1]) / 4), np.log(float(top)), 300))).tolist()
    x = np.array(pts + mids + sub + near_top + wide + [0.0], dtype=np.float32)
    x = np.concatenate([x, -x])
    r = rng.integers(0, 65536, size=x.size).astype(np.uint32)
    got_rne = o.round_em(x, E, M)
    got_sr = o.round_em(x, E, M, r)
    for i, xv in enumerate(x.tolist()):
        a = abs(Fraction(xv))
        if a >= top:
            want_rne = want_sr = top
        else:
            k = bisect.bisect_right(gv, a) - 1                                 # gv[k] <= a < gv[k + 1]
            lo, hi = gv[k], gv[k + 1]
            frac = (a - lo) / (hi - lo)
            want_rne = hi if (frac > Fraction(1, 2) or (frac == Fraction(1, 2) and grid[k][1] == 1)) else lo
            want_sr = hi if (int(frac * 65536) + int(r[i]) >= 65536) else lo
        for name, got, want in (("nearest", got_rne[i], want_rne), ("stochastic", got_sr[i], want_sr)):
            assert Fraction(float(abs(got))) == want, (E, M, name, xv, float(got), float(want))
            assert np.signbit(got) == np.signbit(np.float32(xv))


def test_update_rows_tracks_the_true_sum_over_many_steps_with_compensation():
    """The update rule itself (not only the stand-alone Kahan stream) over 300 steps of the same
    small gradient: without compensation round-to-nearest cancels every step (Section 4.1); with the
    BF16 compensation the pair w - c follows w0 - n lr g, for BF16 and for E4M3 weights, under
    nearest and under stochastic rounding."""
    n_steps, lr = 300, 0.05
    for fmt, w0, g in ((o.BF16, 1.0, 2.0**-6), (o.E4M3, 0.25, 2.0**-4)):      # lr g = 1/10 of a spacing (BF16), 1/10 (E4M3)
        elem = np.arange(8, dtype=np.int64)
        dW = np.full(8, g)
        W0 = o.quantize(np.full(8, w0, np.float32), fmt)
        Wp = W0.copy()
        for s in range(20):
            Wp, _ = o.update_rows(Wp, None, dW, lr, fmt, 0, 0, s, elem)
        assert np.array_equal(Wp, W0)                                          # cancelled every time
        for flags in (o.FLAG_KAHAN, o.FLAG_KAHAN | o.FLAG_SR):
            W, C = W0.copy(), np.zeros(8, np.uint16)
            for s in range(n_steps):
                W, C = o.update_rows(W, C, dW, lr, fmt, flags, 3, s, elem)
            true = w0 - n_steps * lr * g
            est = o.decode(W, fmt).astype(np.float64) - o.decode_bf16(C).astype(np.float64)
            spacing = {o.BF16: 2.0**-7, o.E4M3: 2.0**-3}[fmt] * 2.0 ** np.floor(np.log2(abs(true)))
            assert np.all(np.abs(o.decode(W, fmt) - true) <= spacing)            # w itself within one spacing
            # c is itself held in BF16: every step loses up to half a unit of c, i.e. 2^-9 (nearest; |c| <= spacing / 2) or
            # 2^-8 (stochastic; |c| <= spacing) of a spacing, adding up like a random walk over the 300 steps
            bound = spacing * (2.0**-3 if flags & o.FLAG_SR else 2.0**-5)
            assert np.all(np.abs(est - true) <= bound), (fmt, flags, est, true)
