"""Pins for the CPU oracle: every check here rests on something other than the oracle's own
formulas -- brute force with Python sets / exact rationals, numpy library routines, closed-form
bounds, hand-computed byte patterns, and special cases that reduce to a textbook result.

Citations are to Check-N-Run (arXiv 2010.08679): Section 5.1.1 (tracking bit-vector),
Section 5.1 (incremental view, intermittent policy), Section 5.2 Approach 1 (uniform
quantization F_Q, de-quantization), Approach 3 (greedy range search), Section 6.3.1 (policy
behaviour on the production trace).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle as O

BITS = (2, 3, 4, 8)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers (independent of oracle)

def nearest_grid_sq_error(x, lo, hi, bits):
    """Squared distance of each x_j to the nearest of the 2^b evenly spaced points of [lo, hi],
    in exact rational arithmetic.  This is the definition of uniform quantization with clipping,
    written without any clip / divide / round step."""
    qmax = (1 << bits) - 1
    lo_f, hi_f = Fraction(float(lo)), Fraction(float(hi))
    grid = [lo_f + (hi_f - lo_f) * q / qmax for q in range(qmax + 1)]
    tot = Fraction(0)
    for v in x:
        vf = Fraction(float(v))
        tot += min((vf - g) ** 2 for g in grid)
    return tot


def ulp32(v):
    v = np.float32(abs(v))
    return float(np.spacing(v))


# ------------------------------------------------------------------ tracking (Section 5.1.1)

@pytest.mark.parametrize("n_rows", [1, 31, 32, 33, 64, 1000, 4097])
@pytest.mark.parametrize("dtype", [np.int32, np.int64])
def test_mark_matches_set_bruteforce(n_rows, dtype):
    rng = np.random.default_rng(n_rows)
    idx = rng.integers(-3, n_rows + 3, size=5 * n_rows + 7).astype(dtype)
    bm = O.new_bitmap(n_rows)
    skipped = O.mark_touched(bm, n_rows, idx)
    want = {int(i) for i in idx if 0 <= i < n_rows}
    got = {r for r in range(n_rows) if (int(bm[r >> 5]) >> (r & 31)) & 1}
    assert got == want
    assert skipped == int(np.sum((idx < 0) | (idx >= n_rows)))
    # popcount == number of distinct in-range rows; padding bits stay clear
    assert sum(bin(int(w)).count("1") for w in bm) == len(want)
    if n_rows % 32:
        assert int(bm[-1]) >> (n_rows % 32) == 0


def test_mark_idempotent_and_union():
    n_rows = 5000
    rng = np.random.default_rng(1)
    a = rng.integers(0, n_rows, 3000).astype(np.int64)
    b = rng.integers(0, n_rows, 2000).astype(np.int64)
    bm_a, bm_b, bm_ab = O.new_bitmap(n_rows), O.new_bitmap(n_rows), O.new_bitmap(n_rows)
    O.mark_touched(bm_a, n_rows, a)
    once = bm_a.copy()
    O.mark_touched(bm_a, n_rows, a)
    assert np.array_equal(bm_a, once)                       # idempotent
    O.mark_touched(bm_b, n_rows, b)
    O.mark_touched(bm_ab, n_rows, np.concatenate([a, b]))
    assert np.array_equal(bm_ab, bm_a | bm_b)               # accumulates as a union
    O.clear(bm_ab, n_rows)
    assert not bm_ab.any()


def test_bitvector_footprint_below_paper_bound():
    # Section 5.1.1: the bit-vector is "typically less than 0.05%" of the tables.  One bit per
    # fp32 vector of dimension >= 64 is 1 / (64 * 32) = 0.0488 %.
    for n_rows, dim in [(100_000, 64), (5_000_000, 64), (40_000_000, 128)]:
        frac = O.bitmap_words(n_rows) * 4 / (n_rows * dim * 4)
        assert frac < 0.0005
    assert O.bitmap_words(0) == 0 and O.bitmap_words(1) == 1
    assert O.bitmap_words(32) == 1 and O.bitmap_words(33) == 2


# ------------------------------------------------------------------ incremental view (Section 5.1)

@pytest.mark.parametrize("n_rows", [1, 31, 32, 33, 100, 4096, 10007])
def test_compact_equals_sorted_unique(n_rows):
    rng = np.random.default_rng(7 + n_rows)
    idx = rng.integers(0, n_rows, size=max(1, n_rows // 3)).astype(np.int64)
    bm = O.new_bitmap(n_rows)
    O.mark_touched(bm, n_rows, idx)
    ids, n = O.compact_dirty(bm, n_rows)
    want = np.unique(idx).astype(np.uint32)
    assert n == want.size and np.array_equal(ids, want)
    assert np.all(np.diff(ids.astype(np.int64)) > 0)


def test_compact_empty_full_and_capacity():
    n_rows = 1000
    bm = O.new_bitmap(n_rows)
    ids, n = O.compact_dirty(bm, n_rows)
    assert n == 0 and ids.size == 0
    O.mark_touched(bm, n_rows, np.arange(n_rows, dtype=np.int64))
    ids, n = O.compact_dirty(bm, n_rows)
    assert n == n_rows and np.array_equal(ids, np.arange(n_rows, dtype=np.uint32))
    ids, n = O.compact_dirty(bm, n_rows, capacity=10)
    assert n == n_rows and np.array_equal(ids, np.arange(10, dtype=np.uint32))


# ------------------------------------------------------------------ row range

def test_row_range_equals_numpy_minmax():
    rng = np.random.default_rng(3)
    t = rng.normal(0, 0.05, size=(300, 64)).astype(np.float32)
    ids = rng.permutation(300)[:120].astype(np.uint32)
    out = O.quantize_rows(t, ids, 4)
    assert np.array_equal(out["row_min"], t[ids].min(axis=1))
    assert np.array_equal(out["row_max"], t[ids].max(axis=1))
    assert np.array_equal(out["bias"], out["row_min"])


def test_negative_zero_is_canonicalised():
    t = np.array([[-0.0, -1.0, -0.0, -2.0], [1.0, -0.0, 2.0, 3.0]], dtype=np.float32)
    out = O.quantize_rows(t, None, 4)
    assert out["row_max"][0] == 0.0 and not np.signbit(out["row_max"][0])
    assert out["row_min"][1] == 0.0 and not np.signbit(out["row_min"][1])


# ------------------------------------------------------------------ F_Q (Section 5.2, Approach 1)

@pytest.mark.parametrize("bits", BITS)
def test_scale_closed_form_and_code_invariants(bits):
    rng = np.random.default_rng(bits)
    t = rng.normal(0, 0.05, size=(400, 64)).astype(np.float32)
    out = O.quantize_rows(t, None, bits)
    qmax = (1 << bits) - 1
    lo = out["bias"].astype(np.float64)
    hi = out["row_max"].astype(np.float64)
    exact = (hi - lo) / qmax
    for s, e in zip(out["scale"], exact):
        assert abs(float(s) - e) <= ulp32(e)              # scale = (x_max - x_min)/(2^N - 1)
    codes = out["codes"]
    assert codes.min() >= 0 and codes.max() <= qmax         # codes in [0, 2^N - 1]
    rows = np.arange(t.shape[0])
    assert np.all(codes[rows, t.argmin(axis=1)] == 0)       # the minimum maps to code 0
    assert np.all(codes[rows, t.argmax(axis=1)] == qmax)    # the maximum maps to 2^N - 1


@pytest.mark.parametrize("bits", BITS)
def test_error_bound_half_scale_and_value_range(bits):
    rng = np.random.default_rng(10 + bits)
    t = rng.normal(0, 0.05, size=(400, 128)).astype(np.float32)
    out = O.quantize_rows(t, None, bits)
    deq = O.dequantize(out["codes"], out["scale"], out["bias"])
    scale = out["scale"].astype(np.float64)[:, None]
    mag = np.maximum(np.abs(out["row_min"]), np.abs(out["row_max"])).astype(np.float64)[:, None]
    slack = 4 * np.spacing(mag.astype(np.float32)).astype(np.float64)
    err = np.abs(t.astype(np.float64) - deq.astype(np.float64))
    assert np.all(err <= scale / 2 + slack)                 # worst case scale/2 per element
    l2, mean = O.row_l2(t, deq)
    assert np.all(l2 <= np.sqrt(t.shape[1]) * (scale[:, 0] / 2 + slack[:, 0]))
    # de-quantized values stay inside [min, max]: code 0 gives min exactly, the top code may
    # overshoot max by the few roundings of scale, scale * q and the final addition
    assert np.all(deq >= out["row_min"][:, None])
    assert np.all(deq.astype(np.float64) <= out["row_max"].astype(np.float64)[:, None] + slack)


@pytest.mark.parametrize("bits", BITS)
def test_codes_equal_nearest_grid_point_bruteforce(bits):
    rng = np.random.default_rng(20 + bits)
    t = rng.normal(0, 1.0, size=(40, 8)).astype(np.float32)
    out = O.quantize_rows(t, None, bits)
    qmax = (1 << bits) - 1
    for r in range(t.shape[0]):
        s, b = float(out["scale"][r]), float(out["bias"][r])
        grid = b + s * np.arange(qmax + 1, dtype=np.float64)
        for j in range(t.shape[1]):
            d = np.abs(float(t[r, j]) - grid)
            best = int(np.argmin(d))
            got = int(out["codes"][r, j])
            if got != best:                                  # only allowed at a (near) tie
                assert abs(got - best) == 1
                assert abs(d[got] - d[best]) <= 8 * ulp32(t[r, j])


@pytest.mark.parametrize("bits", BITS)
def test_on_grid_rows_roundtrip_losslessly(bits):
    qmax = (1 << bits) - 1
    rng = np.random.default_rng(30 + bits)
    for step in (2.0 ** -7, 2.0 ** 3):
        for lo in (-1.5, 0.0, 0.625):
            k = rng.integers(0, qmax + 1, size=(50, 32))
            k[:, 0], k[:, 1] = 0, qmax
            t = (lo + step * k).astype(np.float32)
            out = O.quantize_rows(t, None, bits)
            assert np.array_equal(out["codes"], k.astype(np.uint8))
            assert np.all(out["scale"] == np.float32(step))
            assert np.array_equal(O.dequantize(out["codes"], out["scale"], out["bias"]), t)


def test_constant_row_has_zero_scale_and_restores_exactly():
    t = np.full((3, 16), 0.375, dtype=np.float32)
    t[1] = -2.5
    t[2] = 0.0
    for bits in BITS:
        out = O.quantize_rows(t, None, bits)
        assert np.all(out["scale"] == 0) and np.all(out["codes"] == 0)
        assert np.array_equal(O.dequantize(out["codes"], out["scale"], out["bias"]), t)


def test_round_half_to_even_at_exact_ties():
    # lo = 0, hi = 3 at 2 bits -> scale 1; x = 0.5, 1.5, 2.5 sit exactly between grid points.
    t = np.array([[0.0, 3.0, 0.5, 1.5, 2.5, 1.0, 2.0, 0.25]], dtype=np.float32)
    out = O.quantize_rows(t, None, 2)
    assert out["scale"][0] == 1.0
    assert out["codes"][0].tolist() == [0, 3, 0, 2, 2, 1, 2, 0]


def test_asymmetric_beats_symmetric_and_error_falls_with_bits():
    # Section 5.2: asymmetric consistently outperforms symmetric on skewed vectors; Section
    # 6.2.1: more bits, less loss.
    rng = np.random.default_rng(5)
    t = (rng.gamma(2.0, 0.02, size=(500, 64)) - 0.01).astype(np.float32)
    prev = None
    for bits in BITS:
        e = {}
        for mode in (O.RANGE_MINMAX, O.RANGE_SYMMETRIC):
            out = O.quantize_rows(t, None, bits, mode=mode)
            _, e[mode] = O.row_l2(t, O.dequantize(out["codes"], out["scale"], out["bias"]))
        assert e[O.RANGE_MINMAX] < e[O.RANGE_SYMMETRIC]
        if prev is not None:
            assert e[O.RANGE_MINMAX] < prev
        prev = e[O.RANGE_MINMAX]


def test_symmetric_range_is_plus_minus_max_abs():
    rng = np.random.default_rng(6)
    t = rng.normal(0.3, 1.0, size=(50, 16)).astype(np.float32)
    out = O.quantize_rows(t, None, 4, mode=O.RANGE_SYMMETRIC)
    a = np.abs(t).max(axis=1)
    assert np.array_equal(out["bias"], -a)
    exact = 2.0 * a.astype(np.float64) / 15
    assert np.all(np.abs(out["scale"] - exact) <= np.spacing(exact.astype(np.float32)))


# ------------------------------------------------------------------ dense packing

def _golden_patterns():
    with open(os.path.join(GOLDEN, "pack_patterns.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            b, codes, by = [p.strip() for p in line.split("|")]
            yield int(b), [int(c) for c in codes.split()], bytes(int(h, 16) for h in by.split())


def test_pack_hand_computed_byte_patterns():
    n = 0
    for bits, codes, want in _golden_patterns():
        if len(codes) * bits % 8:
            continue
        got = O.pack(np.array([codes], dtype=np.uint8), bits)
        assert bytes(got[0]) == want, (bits, codes)
        assert O.unpack(got, len(codes), bits)[0].tolist() == codes
        n += 1
    assert n >= 8


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("dim", [8, 64, 128, 200])
def test_pack_equals_numpy_packbits_and_roundtrips(bits, dim):
    rng = np.random.default_rng(bits * 1000 + dim)
    codes = rng.integers(0, 1 << bits, size=(37, dim)).astype(np.uint8)
    packed = O.pack(codes, bits)
    assert packed.shape == (37, dim * bits // 8) == (37, O.packed_row_bytes(dim, bits))
    stream = ((codes[:, :, None] >> np.arange(bits)) & 1).astype(np.uint8).reshape(37, dim * bits)
    assert np.array_equal(packed, np.packbits(stream, axis=1, bitorder="little"))
    assert np.array_equal(O.unpack(packed, dim, bits), codes)


def test_pack_rejects_ragged_rows():
    with pytest.raises(ValueError):
        O.pack(np.zeros((1, 3), dtype=np.uint8), 3)      # 9 bits: not a whole number of bytes


# ------------------------------------------------------------------ de-quantize / restore

@pytest.mark.parametrize("bits", BITS)
def test_restore_is_mul_then_add_and_leaves_other_rows(bits):
    rng = np.random.default_rng(40 + bits)
    n_rows, dim = 500, 64
    t = rng.normal(0, 0.05, size=(n_rows, dim)).astype(np.float32)
    ids = np.sort(rng.permutation(n_rows)[:173]).astype(np.uint32)
    out = O.quantize_rows(t, ids, bits)
    packed = O.pack(out["codes"], bits)
    stale = rng.normal(0, 1, size=(n_rows, dim)).astype(np.float32)
    restored = stale.copy()
    O.restore_rows(restored, ids, bits, packed, out["scale"], out["bias"])
    # x = scale * x_q + zero_point with one rounding per operation (numpy fp32 ops)
    want = out["scale"][:, None] * out["codes"].astype(np.float32)
    want = want + out["bias"][:, None]
    assert want.dtype == np.float32
    assert np.array_equal(restored[ids], want)
    others = np.setdiff1d(np.arange(n_rows), ids)
    assert np.array_equal(restored[others], stale[others])
    # encoding the restored rows with the same range reproduces the codes (up to boundary cases)
    again = O.quantize_rows(restored, ids, bits)
    assert np.mean(again["codes"] != out["codes"]) < 1e-3


def test_row_l2_matches_numpy_norm():
    rng = np.random.default_rng(9)
    a = rng.normal(size=(64, 33)).astype(np.float32)
    b = rng.normal(size=(64, 33)).astype(np.float32)
    err, mean = O.row_l2(a, b)
    want = np.linalg.norm(a.astype(np.float64) - b.astype(np.float64), axis=1)
    assert np.allclose(err, want, rtol=1e-14, atol=0)
    assert mean == pytest.approx(want.mean(), rel=1e-14)


# ------------------------------------------------------------------ greedy range (Approach 3)

def test_greedy_iteration_count_reading():
    # ratio bounds the part of the original range that is walked; the range is never collapsed.
    assert O.greedy_iterations(25, 0.6) == 15
    assert O.greedy_iterations(25, 1.0) == 24
    assert O.greedy_iterations(45, 1.0) == 44
    assert O.greedy_iterations(100, 1.0) == 99
    assert O.greedy_iterations(100, 0.5) == 50
    assert O.greedy_iterations(100, 0.0) == 0
    assert O.greedy_iterations(10, 0.05) == 1
    assert O.greedy_iterations(1, 1.0) == 0 and O.greedy_iterations(0, 1.0) == 0


@pytest.mark.parametrize("bits", (2, 3, 4))
def test_greedy_with_zero_ratio_is_plain_minmax(bits):
    rng = np.random.default_rng(50 + bits)
    t = rng.normal(0, 0.05, size=(100, 64)).astype(np.float32)
    a = O.quantize_rows(t, None, bits)
    g = O.quantize_rows(t, None, bits, mode=O.RANGE_GREEDY, num_bins=40, ratio=0.0)
    for k in ("scale", "bias", "codes", "row_min", "row_max"):
        assert np.array_equal(a[k], g[k])


def test_sq_error_equals_nearest_grid_definition():
    rng = np.random.default_rng(60)
    for bits in (2, 3, 4):
        x = rng.normal(0, 1, size=24).astype(np.float32)
        for lo, hi in [(x.min(), x.max()), (-0.5, 0.75), (0.1, 2.0)]:
            lo, hi = np.float32(lo), np.float32(hi)
            got = O.fq_sq_error(x, lo, hi, bits)
            want = float(nearest_grid_sq_error(x, lo, hi, bits))
            assert got == pytest.approx(want, rel=2e-5)


def _lattice_optimum(x, bits, num_bins, n_iter):
    """Smallest nearest-grid error over every range reachable by n_iter or fewer shrink steps."""
    X_min, X_max = Fraction(float(x.min())), Fraction(float(x.max()))
    step = (X_max - X_min) / num_bins
    best = None
    for i in range(n_iter + 1):
        for j in range(n_iter + 1 - i):
            e = nearest_grid_sq_error(x, float(X_min + i * step), float(X_max - j * step), bits)
            best = e if best is None or e < best else best
    return float(best)


@pytest.mark.parametrize("bits", (2, 3, 4))
def test_greedy_sandwiched_between_lattice_optimum_and_minmax(bits):
    rng = np.random.default_rng(70 + bits)
    num_bins, ratio = 12, 1.0
    n_iter = O.greedy_iterations(num_bins, ratio)
    for trial in range(6):
        x = rng.normal(0, 0.02, size=(1, 16)).astype(np.float32)
        x[0, rng.integers(16)] += np.float32(0.3 * (1 if trial % 2 else -1))
        plain = O.quantize_rows(x, None, bits)
        g = O.quantize_rows(x, None, bits, mode=O.RANGE_GREEDY, num_bins=num_bins, ratio=ratio)
        e_plain = float(nearest_grid_sq_error(x[0], plain["bias"][0], plain["row_max"][0], bits))
        lo = g["bias"][0]
        hi_exact = Fraction(float(lo)) + Fraction(float(g["scale"][0])) * ((1 << bits) - 1)
        e_greedy = float(nearest_grid_sq_error(x[0], lo, float(hi_exact), bits))
        e_opt = _lattice_optimum(x[0], bits, num_bins, n_iter)
        tol = 1e-4 * e_plain
        assert e_opt <= e_greedy + tol
        assert e_greedy <= e_plain + tol
        # the chosen range never leaves the original one
        assert lo >= plain["row_min"][0]
        assert float(hi_exact) <= float(plain["row_max"][0]) * (1 + 1e-6) + 1e-12
        # min / max outputs still report the un-shrunk range
        assert g["row_min"][0] == plain["row_min"][0] and g["row_max"][0] == plain["row_max"][0]


def test_greedy_follows_an_independently_evaluated_path():
    # Walk the greedy steps with the nearest-grid error in exact arithmetic (bounds accumulated
    # in fp32 like the text's x_min + step_size) and compare the final range.
    rng = np.random.default_rng(81)
    bits, num_bins, ratio = 3, 10, 0.7
    n_iter = O.greedy_iterations(num_bins, ratio)
    agree = 0
    for trial in range(12):
        x = rng.normal(0, 1.0, size=(1, 12)).astype(np.float32)
        x[0, 0] = np.float32(6.0 + trial)
        X_min, X_max = x.min(), x.max()
        step = np.float32(np.float32(X_max - X_min) / np.float32(num_bins))
        lo, hi = X_min, X_max
        best = (nearest_grid_sq_error(x[0], lo, hi, bits), lo, hi)
        robust = True
        for _ in range(n_iter):
            c_lo, c_hi = np.float32(lo + step), np.float32(hi - step)
            e_lo = nearest_grid_sq_error(x[0], c_lo, hi, bits)
            e_hi = nearest_grid_sq_error(x[0], lo, c_hi, bits)
            if abs(e_lo - e_hi) <= Fraction(1, 10 ** 5) * max(e_lo, e_hi):
                robust = False
            if e_lo < e_hi:
                lo, e = c_lo, e_lo
            else:
                hi, e = c_hi, e_hi
            if abs(e - best[0]) <= Fraction(1, 10 ** 5) * max(e, best[0]):
                robust = False
            if e < best[0]:
                best = (e, lo, hi)
        if not robust:
            continue
        g = O.quantize_rows(x, None, bits, mode=O.RANGE_GREEDY, num_bins=num_bins, ratio=ratio)
        assert g["bias"][0] == best[1]
        want_scale = np.float32(np.float32(best[2] - best[1]) / np.float32((1 << bits) - 1))
        assert g["scale"][0] == want_scale
        agree += 1
    assert agree >= 8


def test_greedy_on_rows_whose_span_is_a_few_float_spacings():
    # Rows that span only a few representable values around a large magnitude: the step is under one
    # spacing, the cumulative bounds move by whole spacings, and late candidate ranges are empty or
    # inverted.  Whatever such candidates score, iteration 0 (the un-shrunk range) is a candidate, so
    # the result can never be worse than plain min/max, the stored range stays inside the row's, and
    # the stored scale is never negative.  Errors are evaluated here with numpy.
    rng = np.random.default_rng(7)
    for mag in (1.0, 1000.0, 3e-3):
        base = np.float32(mag)
        u = np.spacing(base)
        for span in (2, 4, 7, 20, 100):
            x = (base + u * rng.integers(0, span + 1, size=(64, 16)).astype(np.float32)).astype(np.float32)
            x[:, 0], x[:, 1] = base, base + u * span
            for num_bins in (3, 6, 25):
                for bits in (2, 3, 4):
                    g = O.quantize_rows(x, None, bits, mode=O.RANGE_GREEDY, num_bins=num_bins, ratio=1.0)
                    p = O.quantize_rows(x, None, bits)

                    def err(q):
                        # de-quantized as a resume would see it: fp32 product, then fp32 sum (at this
                        # scale the two roundings are the error)
                        back = q["scale"][:, None] * q["codes"].astype(np.float32) + q["bias"][:, None]
                        assert back.dtype == np.float32
                        return np.linalg.norm(x.astype(np.float64) - back.astype(np.float64), axis=1)
                    assert np.all(g["scale"] >= 0)
                    assert np.all(g["bias"] >= p["row_min"])
                    hi = g["bias"].astype(np.float64) + g["scale"].astype(np.float64) * ((1 << bits) - 1)
                    assert np.all(hi <= p["row_max"].astype(np.float64) + u)
                    assert np.all(err(g) <= err(p) * (1 + 1e-9))


def test_greedy_beats_minmax_on_outlier_rows_more_at_low_bits():
    # Approach 3's motivation: one element of large magnitude inflates the scale.  Section 5.2
    # also reports a larger gain at lower bit-widths.
    rng = np.random.default_rng(90)
    t = rng.normal(0, 0.02, size=(200, 64)).astype(np.float32)
    t[np.arange(200), rng.integers(0, 64, 200)] = rng.choice([-1.0, 1.0], 200).astype(np.float32)
    gain = {}
    for bits in (2, 3, 4):
        a = O.quantize_rows(t, None, bits)
        g = O.quantize_rows(t, None, bits, mode=O.RANGE_GREEDY, num_bins=25, ratio=1.0)
        ea, _ = O.row_l2(t, O.dequantize(a["codes"], a["scale"], a["bias"]))
        eg, _ = O.row_l2(t, O.dequantize(g["codes"], g["scale"], g["bias"]))
        assert np.all(eg <= ea * (1 + 1e-6))
        assert np.mean(eg < ea) > 0.8
        gain[bits] = 1.0 - eg.mean() / ea.mean()
    assert gain[2] > 0 and gain[3] > 0 and gain[4] > 0


def test_threads_do_not_change_results():
    rng = np.random.default_rng(100)
    t = rng.normal(0, 0.05, size=(1000, 64)).astype(np.float32)
    ids = np.sort(rng.permutation(1000)[:333]).astype(np.uint32)
    a = O.quantize_rows(t, ids, 4, mode=O.RANGE_GREEDY, num_bins=20, ratio=1.0, n_threads=1)
    b = O.quantize_rows(t, ids, 4, mode=O.RANGE_GREEDY, num_bins=20, ratio=1.0, n_threads=5)
    for k in a:
        assert np.array_equal(a[k], b[k])


# ------------------------------------------------------------------ intermittent policy (Section 5.1)

def test_intermittent_policy_inequality():
    assert not O.full_checkpoint_due([])
    assert not O.full_checkpoint_due([0.25])               # F_c = 1.25 > I_c = 0.5
    assert O.full_checkpoint_due([0.5, 0.8])               # F_c = 2.3 <= I_c = 2.4
    assert not O.full_checkpoint_due([0.5, 0.7])           # F_c = 2.2 >  I_c = 2.1
    assert O.full_checkpoint_due([1.0])                    # F_c = 2 <= I_c = 2 (equality counts)


def test_intermittent_policy_switches_at_interval_eight_on_paper_like_growth():
    # Section 6.3.1: one-shot incrementals start near 25 % of the model, pass 50 % after ten
    # intervals, and the intermittent policy takes a full checkpoint at interval 8, just before
    # the size reaches 50 %.  Linear growth 25 % -> 52 % reproduces that switch point.
    S = [0.25 + 0.03 * k for k in range(12)]
    first = next(i for i in range(1, 12) if O.full_checkpoint_due(S[:i]))
    assert first + 1 == 8 and S[first - 1] < 0.5


# ------------------------------------------------------------------ parameter selection (Section 5.2)

def test_taper_rule_keeps_the_smallest_value_near_the_best():
    grid = [5, 10, 15, 20, 25]
    naive = 1.0
    errs = [0.90, 0.80, 0.712, 0.70, 0.70]                 # improvements .10 .20 .288 .30 .30
    assert O.taper_choice(grid, errs, naive, 0.05) == 15   # .288 >= .95 * .30
    assert O.taper_choice(grid, errs, naive, 0.0) == 20
    assert O.taper_choice(grid, [1.0] * 5, naive, 0.05) == 5    # no improvement at all


def test_selection_never_worse_than_naive_and_sample_agrees_with_full():
    # Section 5.2: the error of the adaptive range is never above the naive one, and the choice made
    # on a small uniform sample matched the choice made on the full checkpoint.
    rng = np.random.default_rng(11)
    t = rng.normal(0, 0.02, size=(6000, 64)).astype(np.float32)
    mask = rng.random(t.shape) < 0.01
    t[mask] = rng.laplace(0, 0.2, size=int(mask.sum())).astype(np.float32)
    bins, ratios = (5, 15, 25, 35, 45), (0.2, 0.4, 0.6, 0.8, 1.0)
    full, rep_full = O.select_greedy_params(t, 4, bins, ratios, n_threads=8)
    for key, e in rep_full.items():
        assert e <= rep_full["naive"] * (1 + 1e-12), key
    sample = t[np.sort(rng.integers(0, t.shape[0], 1500))]
    small, rep_small = O.select_greedy_params(sample, 4, bins, ratios, n_threads=8)
    # the sampled error curve tracks the full one, so the choice lands on the same plateau: at most
    # one grid step away, and as good on the full data as the taper rule demands
    for key in rep_full:
        assert rep_small[key] == pytest.approx(rep_full[key], rel=0.05)
    assert abs(bins.index(small[0]) - bins.index(full[0])) <= 1
    gain = lambda nb: 1.0 - rep_full[("bins", nb)] / rep_full["naive"]  # noqa: E731
    assert gain(small[0]) >= 0.9 * max(gain(nb) for nb in bins)


# ------------------------------------------------------------------ dynamic bit-width selection (Section 6.2.1)

def test_bit_width_follows_the_resume_counts_the_paper_reports():
    # Section 6.2.1: a 2-bit checkpoint survives one resume but not two, 3 bits up to 3 resumes,
    # 4 bits up to 20, 8 bits more than 100; the narrowest width that survives is taken
    assert [O.select_bits(e) for e in (0, 1)] == [2, 2]
    assert [O.select_bits(e) for e in (2, 3)] == [3, 3]
    assert [O.select_bits(e) for e in (4, 10, 20)] == [4, 4, 4]
    assert [O.select_bits(e) for e in (21, 100, 1000)] == [8, 8, 8]
    widths = [O.select_bits(e) for e in range(0, 200)]
    assert widths == sorted(widths) and set(widths) == {2, 3, 4, 8}


def test_bit_width_falls_back_to_eight_bits_when_failures_exceed_the_estimate():
    assert O.select_bits(1, 1) == 2 and O.select_bits(1, 2) == 8
    assert O.select_bits(3, 3) == 3 and O.select_bits(3, 4) == 8
    assert O.select_bits(20, 20) == 4 and O.select_bits(20, 21) == 8
    assert O.select_bits(50, 51) == 8
