"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each one ties a part of
oracle/fb4_oracle.c to something other than itself: hand-worked fixtures,
closed forms, exact brute force in rational arithmetic on tiny blocks,
textbook special cases and invariants of the format (Sec. 3.1-3.4).
"""

import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from fb4_inputs import (DEFAULT_FORMATBOOK, E2M1_X2_FORMATBOOK, UNIFORM_STEP2_FORMATBOOK,
                        range_buckets, synth)
from oracle import fb4_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- helpers
def f2b(a):
    """float32 -> bf16 bit patterns, round to nearest even."""
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def b2f(bits):
    """bf16 bit patterns -> float64 (IEEE value)."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    with np.errstate(invalid="ignore"):          # (signalling NaN patterns)
        return u.view(np.float32).astype(np.float64)


def exact(bits):
    """bf16 bit pattern -> Fraction (finite inputs only)."""
    return Fraction(float(b2f(np.array([bits], dtype=np.uint16))[0]))


def unpack(codes):
    """uint8 [rows][cols/2] -> nibbles [rows][cols]."""
    lo = codes & 0xF
    hi = codes >> 4
    return np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or ":" not in line:
                continue
            k, v = line.split(":", 1)
            out[k.strip()] = v.split()
    return out


def pad_block(vals, block=32):
    v = np.zeros(block, dtype=np.float32)
    v[: len(vals)] = vals
    return f2b(v)


# ------------------------------------------------- formatbook (Sec. 3.1, 3.4)
def test_default_formatbook_meets_the_papers_rules():
    fbk = DEFAULT_FORMATBOOK
    assert fbk.shape == (32, 8)                      # 32 dialects, 5-bit DID
    assert O.validate_formatbook(fbk)
    assert (fbk[:, 0] == 0).all()                    # index 0 is magnitude 0 (App. E.1)
    assert (np.diff(fbk.astype(int), axis=1) > 0).all()
    assert fbk.max() <= 15                           # 4-bit unsigned magnitudes
    tops = fbk[:, 7].astype(int)
    assert (tops >= 8).all() and (np.diff(tops) >= 0).all()   # lower DID = narrower range (App. B)
    counts = [len(b) for b in range_buckets(fbk)]
    assert all(c >= 1 for c in counts)               # every range 8..15 covered (rule 1)
    assert counts == sorted(counts) and counts[0] < counts[-1]  # fewer dialects for narrower ranges
    assert len({tuple(r) for r in fbk.tolist()}) == 32
    for b in range_buckets(fbk):
        # rule 2 (densify small magnitudes): some dialect of the range spends at least half of its eight points
        # on 0..4; rule 3 (preserve large magnitudes): some dialect of the range has at least three points in the
        # top third of the range, more than the range's small-dense dialect has there
        small = [int((fbk[d] <= 4).sum()) for d in b]
        large = [int((3 * fbk[d].astype(int) >= 2 * int(fbk[d, 7])).sum()) for d in b]
        assert max(small) >= 4
        assert max(large) >= 3
        assert len(b) >= 2 and large[int(np.argmax(small))] < max(large)


def test_magnitudes_are_exact_in_fp8_e4m3():
    # Sec. 4.5: the normalized integers 0..15 are representable in FP8 e4m3
    v = torch.arange(16, dtype=torch.float32)
    assert torch.equal(v.to(torch.float8_e4m3fn).to(torch.float32), v)


def test_effective_bit_width():
    # Sec. 3.1: 5-bit DID + 5-bit shared exponent per block; Table 1: 4.31 / 4.63
    assert round(4 + 10 / 32, 2) == 4.31
    assert round(4 + 10 / 16, 2) == 4.62 or round(4 + 10 / 16, 3) == 4.625


def test_validate_rejects_bad_formatbooks():
    good = DEFAULT_FORMATBOOK.copy()
    for mutate in (lambda f: f.__setitem__((3, 0), 1),        # index 0 must be 0
                   lambda f: f.__setitem__((5, 4), f[5, 3]),  # not strictly ascending
                   lambda f: f.__setitem__((0, 7), 7),        # top below 8
                   lambda f: f.__setitem__((31, 7), 16)):     # above 15
        bad = good.copy()
        mutate(bad)
        assert not O.validate_formatbook(bad)
    assert not O.validate_formatbook(np.zeros((33, 8), np.uint8))


# -------------------------------------------------------- worked fixtures
def test_hand_worked_block_codes_and_layout():
    g = read_golden("worked_block_e2m1x2.txt")
    x = f2b(np.array([float(v) for v in g["x"]], dtype=np.float32))[None, :]
    assert np.array_equal(b2f(x)[0], np.array([float(v) for v in g["x"]]))  # all representable
    for sel in (O.SEL_SSE, O.SEL_LUT):
        codes, meta = O.quantize(E2M1_X2_FORMATBOOK, x, selector=sel)
        nib = unpack(codes)[0]
        assert (nib & 7).tolist() == [int(v) for v in g["index"]]
        assert (nib >> 3).tolist() == [int(v) for v in g["sign"]]
        assert codes[0].tolist() == [int(v, 16) for v in g["codes"]]
        assert int(meta[0, 0]) == int(g["meta"][0], 16)


def test_hand_worked_lut_selection():
    g = read_golden("worked_lut_selection.txt")
    fbk = np.array([[0, 1, 2, 3, 4, 6, 8, 12], [0, 2, 4, 6, 8, 10, 12, 14]], dtype=np.uint8)
    for blk in ("block1", "block2"):
        x = f2b(np.array([float(v) for v in g[blk + "_x"]], dtype=np.float32))
        cand, scores, did, e = O.block_scores(fbk, x, selector=O.SEL_LUT, num_groups=8)
        assert cand.tolist() == [0, 1]
        assert scores.tolist() == [float(v) for v in g[blk + "_scores"]]
        assert did == int(g[blk + "_did"][0]) and e == 3


# ------------------------------------------------ shared exponent (Sec. 3.1)
def test_exponent_is_floor_log2_of_block_max_and_max_lands_in_8_16(fbk):
    x = synth.bf16_bits(synth.vdit_activation(rows=64, cols=1024, seed=21))
    codes, meta = O.quantize(fbk, x, selector=O.SEL_LUT)
    a = np.abs(b2f(x)).reshape(64, -1, 32).max(axis=2)
    mant, ex = np.frexp(a)                 # a = mant * 2^ex, mant in [0.5,1)
    assert np.array_equal((meta >> 8).astype(int) - 127, ex - 1)
    xhat_max = a * np.exp2(3.0 - (ex - 1))
    assert (xhat_max >= 8).all() and (xhat_max < 16).all()


def test_power_of_two_scaling_shifts_only_the_exponent(fbk):
    x = synth.bf16_bits(synth.gaussian_outlier(rows=32, cols=512, seed=22))
    for sel in (O.SEL_SSE, O.SEL_LUT):
        c0, m0 = O.quantize(fbk, x, selector=sel)
        for k in (-9, 5, 17):
            xs = (x.astype(np.int32) + (k << 7)).astype(np.uint16)   # exponent field + k
            ck, mk = O.quantize(fbk, xs, selector=sel)
            assert np.array_equal(ck, c0)
            assert np.array_equal(mk & 0xFF, m0 & 0xFF)
            assert np.array_equal((mk >> 8).astype(int), (m0 >> 8).astype(int) + k)


def test_exponent_clamps_and_zero_block(fbk):
    tiny = np.full((1, 32), 0x0003, dtype=np.uint16)       # subnormal block
    zero = np.zeros((1, 32), dtype=np.uint16)
    huge = np.full((1, 32), 0x7F7F, dtype=np.uint16)       # largest finite bf16
    inf = zero.copy(); inf[0, 4] = 0x7F80
    for x, e in ((tiny, -123), (zero, -123), (huge, 127), (inf, 127)):
        _, meta = O.quantize(fbk, x, selector=O.SEL_SSE)
        assert int(meta[0, 0] >> 8) - 127 == e
    # every dequantized value is a normal bf16 or zero
    y = O.dequantize(fbk, *O.quantize(fbk, tiny, selector=O.SEL_SSE))
    ef = (y >> 7) & 0xFF
    assert ((ef > 0) | ((y & 0x7FFF) == 0)).all()


# -------------------------------------------- rounding into a dialect (Sec. 3.2)
def test_rounding_matches_midpoint_thresholds_for_every_bf16_value_below_16():
    """Independent formulation: the index is the number of decision boundaries
    (half-way points between neighbouring magnitudes) that the value reaches;
    reaching a boundary exactly counts, i.e. ties go up (Sec. 3.2)."""
    bits = np.arange(0, 0x4180, dtype=np.uint16)            # every bf16 in [0,16)
    vals = b2f(bits)
    assert vals.max() < 16 and b2f(np.array([0x4180], np.uint16))[0] == 16.0
    x = np.zeros((bits.size, 32), dtype=np.uint16)
    x[:, 0] = 0x4100                                        # 8.0 fixes e = 3, xhat = |x|
    x[:, 1] = bits
    x[:, 2] = bits | 0x8000
    for d in range(32):
        one = DEFAULT_FORMATBOOK[d:d + 1]
        codes, meta = O.quantize(one, x, selector=O.SEL_SSE)
        assert ((meta >> 8) == 130).all()
        nib = unpack(codes)
        m = one[0].astype(np.float64)
        bounds = (m[:-1] + m[1:]) / 2.0
        want = (vals[:, None] >= bounds[None, :]).sum(axis=1)
        assert np.array_equal(nib[:, 1] & 7, want)
        assert np.array_equal(nib[:, 2] & 7, want) and (nib[:, 2] >> 3 == 1).all()


def test_uniform_step2_dialect_closed_form():
    rng = np.random.default_rng(5)
    v = rng.uniform(0, 15.4, size=(200, 32)).astype(np.float32)
    v[:, 0] = 15.5
    x = f2b(v)
    xv = b2f(x)
    codes, meta = O.quantize(UNIFORM_STEP2_FORMATBOOK, x, selector=O.SEL_LUT)
    y = O.dequantize(UNIFORM_STEP2_FORMATBOOK, codes, meta, out_dtype=O.OUT_F32)
    want = np.minimum(14.0, 2.0 * np.floor(xv / 2.0 + 0.5))
    assert np.array_equal(y.astype(np.float64), want)


def _e2m1_round(v):
    """Round a non-negative real to the FP4 E2M1 grid by its floating-point
    structure (1 mantissa bit, exponents 0..2, subnormal step 0.5), saturating
    at 6; ties excluded by the caller."""
    if v >= 6:
        return 6.0
    if v < 1:
        return round(v * 2) / 2
    e = min(2, int(math.floor(math.log2(v))))
    step = 2.0 ** (e - 1)
    return round(v / step) * step


def test_one_dialect_e2m1x2_is_mxfp4_with_power_of_two_scale():
    """Sec. 4.5 treats MXFP4 as 'the same power-of-two scaling with FP4': with
    the single dialect 2*{E2M1 values} FB4 is MXFP4 with scale
    2^(floor(log2 max) - 2) and saturation."""
    rng = np.random.default_rng(6)
    v = (rng.standard_t(3, size=(300, 32)) * 3).astype(np.float32)
    x = f2b(v)
    xv = b2f(x)
    codes, meta = O.quantize(E2M1_X2_FORMATBOOK, x, selector=O.SEL_SSE)
    y = O.dequantize(E2M1_X2_FORMATBOOK, codes, meta, out_dtype=O.OUT_F32).astype(np.float64)
    checked = 0
    for r in range(xv.shape[0]):
        scale = 2.0 ** (math.floor(math.log2(np.abs(xv[r]).max())) - 2)
        for i in range(32):
            t = abs(xv[r, i]) / scale
            if t in (0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0):
                continue                                   # on a decision boundary of the E2M1 grid
            assert abs(y[r, i]) == _e2m1_round(t) * scale
            assert (y[r, i] < 0) == (xv[r, i] < 0) or y[r, i] == 0
            checked += 1
    assert checked > 9000


# ---------------------------------------------- exhaustive selection (Sec. 3.2)
def _sse_argmin_exact(fbk, xhat_fracs):
    """argmin over dialects of sum_i min_k (xhat_i - m_k)^2 in exact rational
    arithmetic, lowest DID on ties.  Independent of any tie rule for rounding."""
    best, bests = None, None
    for d, dialect in enumerate(fbk.tolist()):
        s = sum(min((v - m) ** 2 for m in dialect) for v in xhat_fracs)
        if bests is None or s < bests:
            best, bests = d, s
    return best


def test_sse_selection_equals_exact_brute_force_on_tiny_blocks(fbk):
    grid = [0.0, 0.375, 1.0, 2.5, 3.25, 4.5, 5.0, 6.75, 7.0, 9.5, 11.0, 13.25]
    n = 0
    for top in (8.0, 10.5, 15.0):
        for combo in itertools.combinations_with_replacement(grid, 3):
            if max(combo) > top:
                continue
            vals = [top] + list(combo)
            x = pad_block(vals)
            _, _, did, e = O.block_scores(fbk, x, selector=O.SEL_SSE)
            assert e == 3
            assert did == _sse_argmin_exact(fbk, [Fraction(v) for v in vals])
            n += 1
    assert n > 400


def test_sse_selection_equals_exact_brute_force_on_random_blocks(fbk):
    """Full 32-element blocks with tiny elements mixed in: the elements the
    oracle leaves out of its sums (normalized magnitude < 0.5) must not change
    the argmin, ties included."""
    rng = np.random.default_rng(7)
    for t in range(120):
        v = rng.standard_t(3, size=32).astype(np.float32) * (10.0 ** rng.integers(-3, 4))
        if t % 3 == 0:
            v[rng.integers(0, 32, 6)] *= 1e-12
        if t % 4 == 0:
            v = np.round(v)                                  # many exact ties
        x = f2b(v)
        _, _, did, e = O.block_scores(fbk, x, selector=O.SEL_SSE)
        xh = [abs(exact(b)) * Fraction(2) ** (3 - e) for b in x.tolist()]
        assert max(xh) < 16 and (max(xh) >= 8 or max(xh) == 0)
        assert did == _sse_argmin_exact(fbk, xh)


def test_sse_full_selection_is_the_minimum_over_one_dialect_quantizers(fbk):
    x = synth.bf16_bits(synth.vdit_activation(rows=8, cols=512, seed=23))
    xv = b2f(x)
    codes, meta = O.quantize(fbk, x, selector=O.SEL_SSE)
    err = ((xv - O.dequantize(fbk, codes, meta, out_dtype=O.OUT_F32)) ** 2).reshape(8, -1, 32).sum(2)
    per = []
    for d in range(32):
        c, m = O.quantize(fbk[d:d + 1], x, selector=O.SEL_SSE)
        per.append(((xv - O.dequantize(fbk[d:d + 1], c, m, out_dtype=O.OUT_F32)) ** 2)
                   .reshape(8, -1, 32).sum(2))
    per = np.stack(per)
    assert np.allclose(err, per.min(axis=0), rtol=1e-12, atol=0)
    assert np.array_equal(meta & 0xFF, per.argmin(axis=0))    # argmin takes the first minimum


def test_sse_selection_ignores_element_order_lut_g8_does_not(fbk):
    rng = np.random.default_rng(8)
    x = synth.bf16_bits(synth.gaussian_outlier(rows=16, cols=1024, seed=24))
    xb = x.reshape(-1, 32)
    perm = rng.permutation(32)
    d_sse = O.quantize(fbk, xb, selector=O.SEL_SSE)[1] & 0xFF
    d_sse_p = O.quantize(fbk, np.ascontiguousarray(xb[:, perm]), selector=O.SEL_SSE)[1] & 0xFF
    assert np.array_equal(d_sse, d_sse_p)
    d32 = O.quantize(fbk, xb, selector=O.SEL_LUT, num_groups=32)[1] & 0xFF
    d32_p = O.quantize(fbk, np.ascontiguousarray(xb[:, perm]), selector=O.SEL_LUT, num_groups=32)[1] & 0xFF
    assert np.array_equal(d32, d32_p)                        # g = block scores every element
    d8 = O.quantize(fbk, xb, selector=O.SEL_LUT, num_groups=8)[1] & 0xFF
    d8_p = O.quantize(fbk, np.ascontiguousarray(xb[:, perm]), selector=O.SEL_LUT, num_groups=8)[1] & 0xFF
    assert (d8 != d8_p).any()                                # group maxima depend on the partition
    inside = np.concatenate([rng.permutation(4) + 4 * j for j in range(8)])
    d8_i = O.quantize(fbk, np.ascontiguousarray(xb[:, inside]), selector=O.SEL_LUT, num_groups=8)[1] & 0xFF
    assert np.array_equal(d8, d8_i)                          # ...but not on order inside a group


# -------------------------------------------- the paper's online rule (Sec. 3.2)
def _abs_err_exact(dialect, v):
    return min(abs(v - m) for m in dialect)


def test_lut_score_is_within_a_quarter_per_group_of_the_exact_absolute_error(fbk):
    """The bin midpoint stands in for a value at most 0.25 away (0.5-wide
    bins), and distance to a fixed set is 1-Lipschitz, so per group the
    approximate error is within 0.25 of the exact absolute error of the
    group's maximum."""
    rng = np.random.default_rng(9)
    for g in (8, 32):
        for t in range(40):
            x = f2b(rng.standard_t(3, size=32).astype(np.float32) * 4)
            cand, scores, did, e = O.block_scores(fbk, x, selector=O.SEL_LUT, num_groups=g)
            xh = [abs(exact(b)) * Fraction(2) ** (3 - e) for b in x.tolist()]
            per = 32 // g
            umax = [max(xh[j * per:(j + 1) * per]) for j in range(g)]
            for d, s in zip(cand.tolist(), scores.tolist()):
                ex = sum(_abs_err_exact(fbk[d].tolist(), u) for u in umax)
                assert abs(Fraction(s) - ex) <= Fraction(g, 4)
            assert did == cand[int(np.argmin(scores))]        # first minimum = lowest DID


def test_lut_score_is_exact_when_group_maxima_sit_on_bin_midpoints(fbk):
    """Values k/2 + 1/4 are their own bin midpoints, so the rule must return
    the exact L1 error over the group maxima and hence its true argmin."""
    rng = np.random.default_rng(10)
    for g in (8, 32):
        for t in range(60):
            k = rng.integers(0, 32, size=32)
            k[rng.integers(0, 32)] = rng.integers(16, 32)       # block max in [8,16)
            v = k / 2.0 + 0.25
            x = f2b((v * rng.choice([-1.0, 1.0], size=32)).astype(np.float32))
            cand, scores, did, e = O.block_scores(fbk, x, selector=O.SEL_LUT, num_groups=g)
            assert e == 3
            per = 32 // g
            umax = [Fraction(float(v[j * per:(j + 1) * per].max())) for j in range(g)]
            exact_scores = [sum(_abs_err_exact(fbk[d].tolist(), u) for u in umax) for d in range(32)]
            assert [Fraction(s) for s in scores.tolist()] == exact_scores
            assert did == exact_scores.index(min(exact_scores))


def test_lut_groups_are_contiguous(fbk):
    """One large value per contiguous group of four makes every group maximum
    large; under a strided partition some groups would only see small values."""
    v = np.full(32, 0.25, dtype=np.float32)
    v[0:32:4] = [9, 9, 9, 9, 9, 9, 9, 13]
    x = f2b(v)
    _, s_c, _, _ = O.block_scores(fbk[:1], x, selector=O.SEL_LUT, num_groups=8)
    # contiguous: maxima 9 x7 and 13 -> dialect 0 = {..,6,8}: |9.25-8|*7 + |13.25-8|
    assert s_c[0] == 7 * 1.25 + 5.25


# ------------------------------------------------------ codes and signs
def test_codes_are_valid_and_sign_symmetric(fbk):
    x = synth.bf16_bits(synth.vdit_activation(rows=16, cols=1024, seed=25))
    for sel in (O.SEL_SSE, O.SEL_LUT):
        c, m = O.quantize(fbk, x, selector=sel)
        assert ((m & 0xFF) < 32).all()
        cn, mn = O.quantize(fbk, x ^ 0x8000, selector=sel)
        assert np.array_equal(mn, m)
        assert np.array_equal(cn, c ^ 0x88)                   # only the sign bits flip
        y = O.dequantize(fbk, c, m, out_dtype=O.OUT_F32).astype(np.float64)
        did = np.repeat(m & 0xFF, 32, axis=1)
        e = np.repeat((m >> 8).astype(int) - 127, 32, axis=1)
        mag = np.abs(y) / np.exp2(e - 3.0)
        assert (mag == np.round(mag)).all()
        assert all(int(v) in set(fbk[d].tolist()) for v, d in zip(mag.ravel()[:4096], did.ravel()[:4096]))
        # bf16 output is the same number
        yb = O.dequantize(fbk, c, m, out_dtype=O.OUT_BF16)
        assert np.array_equal(b2f(yb), y)
        # sign of the output follows the sign bit of the input, zero included
        assert np.array_equal(yb >> 15, x >> 15)


def test_dequantize_quantize_is_idempotent_with_exhaustive_selection(fbk):
    """A dequantized block is exactly representable again: with the scale
    unchanged its own dialect has zero error; if its largest code fell below 8
    the scale drops by one and the doubled values are even, which the uniform
    step-2 dialect of the default formatbook holds."""
    x = synth.bf16_bits(synth.vdit_activation(rows=16, cols=1024, seed=26))
    y = O.dequantize(fbk, *O.quantize(fbk, x, selector=O.SEL_SSE))
    y2 = O.dequantize(fbk, *O.quantize(fbk, y, selector=O.SEL_SSE))
    assert np.array_equal(y, y2)


def test_quantization_error_is_bounded_by_half_the_largest_gap(fbk):
    x = synth.bf16_bits(synth.gaussian_outlier(rows=16, cols=1024, seed=27))
    xv = b2f(x)
    for sel in (O.SEL_SSE, O.SEL_LUT):
        c, m = O.quantize(fbk, x, selector=sel)
        y = O.dequantize(fbk, c, m, out_dtype=O.OUT_F32).astype(np.float64)
        did = np.repeat(m & 0xFF, 32, axis=1)
        e = np.repeat((m >> 8).astype(int) - 127, 32, axis=1)
        f = fbk.astype(float)
        gap = np.maximum(np.diff(f, axis=1).max(axis=1) / 2, 16 - f[:, 7])   # inside gaps, saturation
        assert (np.abs(xv - y) <= gap[did] * np.exp2(e - 3.0)).all()


def test_nan_and_inf_readings(fbk):
    v = np.linspace(-3, 3, 32).astype(np.float32)
    x = f2b(v)[None, :].copy()
    ref_c, ref_m = O.quantize(fbk, x, selector=O.SEL_SSE)
    xn = x.copy(); xn[0, 5] = 0x7FC0; xn[0, 9] = 0xFFC0
    x0 = x.copy(); x0[0, 5] = 0x0000; x0[0, 9] = 0x8000
    cn, mn = O.quantize(fbk, xn, selector=O.SEL_SSE)
    c0, m0 = O.quantize(fbk, x0, selector=O.SEL_SSE)
    assert np.array_equal(mn, m0) and np.array_equal(cn, c0)   # a NaN behaves like a signed zero
    xi = x.copy(); xi[0, 2] = 0xFF80
    ci, mi = O.quantize(fbk, xi, selector=O.SEL_SSE)
    assert int(mi[0, 0] >> 8) == 254                            # e clamps to 127
    nib = unpack(ci)[0]
    assert nib[2] == 0xF and (np.delete(nib, 2) & 7 == 0).all()  # Inf saturates, the rest vanish


# ------------------------------------------------ decomposition (Sec. 3.3)
def test_decomposition_never_increases_any_elements_error(fbk):
    x = synth.bf16_bits(synth.vdit_activation(rows=48, cols=1024, seed=28))
    xv = b2f(x)
    sal = np.array([0, 3, 4, 17, 40, 47], dtype=np.int32)
    for sel in (O.SEL_SSE, O.SEL_LUT):
        c1, m1 = O.quantize(fbk, x, selector=sel)
        c2, m2 = O.decompose(fbk, x, c1, m1, sal, selector=sel)
        y1 = O.dequantize(fbk, c1, m1, out_dtype=O.OUT_F32).astype(np.float64)
        y12 = O.dequantize(fbk, c1, m1, codes2=c2, meta2=m2, salient_rows=sal,
                           out_dtype=O.OUT_F32).astype(np.float64)
        e1 = np.abs(xv - y1)
        e12 = np.abs(xv - y12)
        # fp32 sum of the two planes can round by half an ulp of the result
        slack = np.abs(y12) * 2.0 ** -24
        assert (e12 <= e1 + slack).all()
        assert (e12[sal] ** 2).sum() < 0.2 * (e1[sal] ** 2).sum()
        rest = np.setdiff1d(np.arange(48), sal)
        assert np.array_equal(y12[rest], y1[rest])              # other rows: plane 1 only
        # plane 2 is the plain quantization of the rounded residual
        delta = f2b((xv[sal] - y1[sal]).astype(np.float32))
        c2b, m2b = O.quantize(fbk, delta, selector=sel)
        assert np.array_equal(c2, c2b) and np.array_equal(m2, m2b)


def test_residual_is_exactly_representable_and_plane_sum_rounds_to_nearest_even(fbk):
    """Zero is in every dialect, so the nearest magnitude is never farther from
    x than x itself: |x - y| <= |x| and the residual, a multiple of x's last
    bit, fits bf16 without rounding.  The sum of the two planes does round:
    the bf16 output must be the round-to-nearest-even of the fp32 output
    (checked against torch's conversion)."""
    x = synth.bf16_bits(synth.vdit_activation(rows=32, cols=1024, seed=34))
    xv = b2f(x)
    sal = np.arange(0, 32, 3, dtype=np.int32)
    for sel in (O.SEL_SSE, O.SEL_LUT):
        c1, m1 = O.quantize(fbk, x, selector=sel)
        y1 = O.dequantize(fbk, c1, m1, out_dtype=O.OUT_F32).astype(np.float64)
        delta = xv - y1
        assert (np.abs(delta) <= np.abs(xv)).all()
        assert np.array_equal(b2f(f2b(delta.astype(np.float32))), delta)
        c2, m2 = O.decompose(fbk, x, c1, m1, sal, selector=sel)
        yf = O.dequantize(fbk, c1, m1, codes2=c2, meta2=m2, salient_rows=sal, out_dtype=O.OUT_F32)
        yb = O.dequantize(fbk, c1, m1, codes2=c2, meta2=m2, salient_rows=sal, out_dtype=O.OUT_BF16)
        want = torch.from_numpy(yf).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(yb, want)
        assert (b2f(yb)[sal] != yf[sal]).any()                 # rounding really happens
        both = y1[sal] + O.dequantize(fbk, c2, m2, out_dtype=O.OUT_F32).astype(np.float64)
        assert np.array_equal(yf[sal], both.astype(np.float32))  # one fp32 rounding of the exact sum


def test_decomposition_of_a_representable_tensor_is_zero(fbk):
    x = synth.bf16_bits(synth.gaussian_outlier(rows=4, cols=256, seed=29))
    y = O.dequantize(fbk, *O.quantize(fbk, x, selector=O.SEL_SSE))
    c1, m1 = O.quantize(fbk, y, selector=O.SEL_SSE)
    sal = np.arange(4, dtype=np.int32)
    c2, m2 = O.decompose(fbk, y, c1, m1, sal, selector=O.SEL_SSE)
    assert (c2 == 0).all() and ((m2 >> 8) == 4).all()          # all +0, exponent at its floor


# ------------------------------------------------------- SeDA (Sec. 3.4)
def test_seda_restricts_the_argmin_to_the_rows_sub_formatbook(fbk):
    x, comp = synth.mixture_activation(rows=64, cols=512, seed=30, n_components=6)
    x = synth.bf16_bits(x)
    sub = synth.seda_sub_formatbooks(fbk, n_groups=6, seed=30)
    tops = fbk[sub.astype(int), 7]
    assert (tops == np.arange(8, 16)[None, :]).all()            # one dialect per dynamic range
    tg = comp.copy()
    tg[::5] = -1                                               # -1 = full formatbook
    for sel, g in ((O.SEL_SSE, 8), (O.SEL_LUT, 8), (O.SEL_LUT, 32)):
        c, m = O.quantize(fbk, x, selector=sel, num_groups=g, token_group=tg, sub_formatbooks=sub)
        cf, mf = O.quantize(fbk, x, selector=sel, num_groups=g)
        did = m & 0xFF
        for r in range(64):
            if tg[r] < 0:
                assert np.array_equal(m[r], mf[r]) and np.array_equal(c[r], cf[r])
                continue
            assert np.isin(did[r], sub[tg[r]]).all()
            for b in range(0, 16, 5):
                cand, scores, _, _ = O.block_scores(fbk, x[r, 32 * b:32 * b + 32], selector=sel, num_groups=g)
                allowed = sub[tg[r]].astype(int)
                s = scores[allowed]
                assert did[r, b] == allowed[int(np.argmin(s))]


def test_seda_with_the_whole_formatbook_as_sub_formatbook_is_plain_quantize():
    fbk8 = DEFAULT_FORMATBOOK[[1, 3, 5, 8, 11, 16, 22, 28]]
    x = synth.bf16_bits(synth.gaussian_outlier(rows=8, cols=256, seed=31))
    sub = np.arange(8, dtype=np.uint8)[None, :]
    tg = np.zeros(8, dtype=np.int32)
    for sel in (O.SEL_SSE, O.SEL_LUT):
        a = O.quantize(fbk8, x, selector=sel, token_group=tg, sub_formatbooks=sub)
        b = O.quantize(fbk8, x, selector=sel)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


# ------------------------------------------- two-stage selection (Sec. 3.2)
def test_two_stage_picks_within_the_range_of_the_block_maximum(fbk):
    x = synth.bf16_bits(synth.vdit_activation(rows=16, cols=1024, seed=32))
    a = np.abs(b2f(x)).reshape(16, -1, 32).max(axis=2)
    for sel in (O.SEL_SSE, O.SEL_LUT):
        c, m = O.quantize(fbk, x, selector=sel, flags=O.FLAG_TWO_STAGE)
        e = (m >> 8).astype(int) - 127
        r = np.floor(a * np.exp2(3.0 - e)).astype(int)
        assert np.array_equal(fbk[(m & 0xFF).astype(int), 7], r)   # every range has a dialect
        for row, b in ((0, 0), (3, 7), (15, 31)):
            cand, scores, did, _ = O.block_scores(fbk, x[row, 32 * b:32 * b + 32], selector=sel)
            allowed = np.nonzero(fbk[:, 7] == r[row, b])[0]
            assert int(m[row, b] & 0xFF) == allowed[int(np.argmin(scores[allowed]))]


def test_block_size_16(fbk):
    x = synth.bf16_bits(synth.gaussian_outlier(rows=8, cols=256, seed=33))
    for sel in (O.SEL_SSE, O.SEL_LUT):
        c16, m16 = O.quantize(fbk, x, block=16, selector=sel)
        assert m16.shape == (8, 16)
        # a row of 16-element blocks equals the same data laid out as 32-element
        # blocks padded with zeros, which change neither scale nor any score
        # (for the online rule: with twice the groups)
        xp = np.zeros((8 * 16, 32), dtype=np.uint16)
        xp[:, :16] = x.reshape(-1, 16)
        c32, m32 = O.quantize(fbk, xp, block=32, selector=sel, num_groups=16)
        # (online rule: the 8 all-zero groups of the padding add the same 0.25 to every dialect's score)
        assert np.array_equal(m16.ravel(), m32.ravel())
        assert np.array_equal(c16.reshape(-1, 8), c32[:, :8])
        assert not c32[:, 8:].any()
    # the online rule's groups at block size 16 are runs of 16 / num_groups elements: 16 groups score every
    # element, so the order inside a block no longer matters, while 8 groups of 2 depend on it
    rng = np.random.default_rng(33)
    perm = np.concatenate([rng.permutation(16) + 16 * b for b in range(16)])
    _, m_all = O.quantize(fbk, x, block=16, selector=O.SEL_LUT, num_groups=16)
    _, m_all_p = O.quantize(fbk, np.ascontiguousarray(x[:, perm]), block=16, selector=O.SEL_LUT, num_groups=16)
    assert np.array_equal(m_all, m_all_p)
    _, m8 = O.quantize(fbk, x, block=16, selector=O.SEL_LUT, num_groups=8)
    _, m8_p = O.quantize(fbk, np.ascontiguousarray(x[:, perm]), block=16, selector=O.SEL_LUT, num_groups=8)
    assert not np.array_equal(m8, m8_p)


def test_hand_worked_lut_selection_block16():
    g = read_golden("worked_lut_selection_block16.txt")
    fbk = np.array([[0, 1, 2, 3, 4, 6, 8, 12], [0, 2, 4, 6, 8, 10, 12, 14]], dtype=np.uint8)
    row = []
    for blk in ("block1", "block2"):
        x = f2b(np.array([float(v) for v in g[blk + "_x"]], dtype=np.float32))
        assert x.size == 16
        cand, scores, did, e = O.block_scores(fbk, x, selector=O.SEL_LUT, num_groups=8)
        assert cand.tolist() == [0, 1]
        assert scores.tolist() == [float(v) for v in g[blk + "_scores"]]
        assert did == int(g[blk + "_did"][0]) and e == 3
        row.append(x)
    # the two blocks side by side as one row of 32 elements quantized with block size 16
    codes, meta = O.quantize(fbk, np.concatenate(row)[None, :], block=16, selector=O.SEL_LUT, num_groups=8)
    assert meta[0].tolist() == [int(g["block1_meta"][0], 16), int(g["block2_meta"][0], 16)]
    assert codes[0, :8].tolist() == [int(v, 16) for v in g["block1_codes"]]
    nib = unpack(codes)[0, :16]
    assert (nib & 7).tolist() == [int(v) for v in g["block1_index"]]
    assert (nib >> 3).tolist() == [int(v) for v in g["block1_sign"]]


# ------------------------------------------------------------ MXFP8 operands
def _mx_value(elems, scales):
    """Decode MXFP8 operands with torch's own FP8 type: E4M3 value * 2^(scale byte - 127)."""
    v = torch.from_numpy(elems.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    s = np.ldexp(1.0, scales.astype(np.int64) - 127)
    return v * np.repeat(s, 32, axis=1)


def test_mxfp8_repack_of_block32_decodes_to_the_same_values(fbk):
    # Sec. 4.5 / App. E.2: magnitudes 0..15 are exact in E4M3 and the scale is a power of two
    x = synth.bf16_bits(synth.vdit_activation(rows=24, cols=512, seed=34))
    c, m = O.quantize(fbk, x)
    el, sc = O.repack_mxfp8(fbk, c, m)
    assert el.shape == (24, 512) and sc.shape == (24, 16)
    y = O.dequantize(fbk, c, m, out_dtype=O.OUT_F32).astype(np.float64)
    assert np.array_equal(_mx_value(el, sc), y)
    # the sign bit travels even when the magnitude is zero (same convention as the codes)
    nib = np.stack([c & 15, c >> 4], axis=2).reshape(24, 512)
    assert np.array_equal(el >> 7, nib >> 3)
    # every element is one of the sixteen integers, so the low mantissa pattern is that of torch's conversion
    mags = torch.arange(16, dtype=torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert set(np.unique(el & 0x7F).tolist()) <= set(mags.tolist())


def test_mxfp8_repack_of_block16_shares_the_larger_exponent(fbk):
    rng = np.random.default_rng(35)
    rows, cols = 16, 256
    # neighbouring 16-element blocks with very different magnitudes: exponent gaps 0..14
    base = rng.standard_normal((rows, cols)).astype(np.float32)
    gap = rng.integers(0, 15, size=(rows, cols // 16))
    x = f2b(base * np.repeat(np.ldexp(1.0, -gap), 16, axis=1).astype(np.float32))
    c, m = O.quantize(fbk, x, block=16)
    el, sc = O.repack_mxfp8(fbk, c, m, block=16)
    eb = (m >> 8).astype(np.int64).reshape(rows, cols // 32, 2)
    assert np.array_equal(sc, (eb.max(axis=2) - 3).astype(np.uint8))
    # each element is torch's round-to-nearest-even E4M3 of (decoded value / MX scale)
    y = O.dequantize(fbk, c, m, block=16, out_dtype=O.OUT_F32).astype(np.float64)
    scale = np.repeat(np.ldexp(1.0, sc.astype(np.int64) - 127), 32, axis=1)
    want = torch.from_numpy((y / scale).astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    nz = (el & 0x7F) != 0
    assert np.array_equal(el[nz], want[nz])
    assert np.array_equal(el & 0x7F, want & 0x7F)
    # exact whenever the two exponents of an MX block differ by at most 9
    close = np.repeat((eb.max(axis=2) - eb.min(axis=2)) <= 9, 32, axis=1)
    assert close.any() and (~close).any()
    assert np.array_equal(_mx_value(el, sc)[close], y[close])


def test_e4m3_rounding_of_the_oracle_on_every_shifted_magnitude():
    # two dialects that together hold every magnitude 0..15; an MX block made of a 16-element block with
    # exponent byte 130 - k and one with 130, k = 0..20: the first block's elements are m * 2^-k in units of
    # the shared scale, compared one by one with torch's conversion (normals, subnormals, ties, underflow)
    fb = np.array([[0, 1, 2, 3, 4, 5, 6, 8], [0, 7, 10, 11, 12, 13, 14, 15]], dtype=np.uint8)
    idx = np.arange(8)
    top = torch.tensor([15.0]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()[0]
    seen = set()
    for k in range(0, 21):
        for did in (0, 1):
            codes = np.zeros((1, 16), dtype=np.uint8)
            codes[0, :8] = (idx | (idx << 4)).astype(np.uint8)           # elements 0..15: every index twice
            codes[0, 8:] = 0x77                                           # elements 16..31: the top magnitude
            meta = np.array([[did | ((130 - k) << 8), 1 | (130 << 8)]], dtype=np.uint16)
            el, sc = O.repack_mxfp8(fb, codes, meta, block=16)
            assert sc[0, 0] == 127
            vals = fb[did][np.repeat(idx, 2)].astype(np.float64) * 2.0 ** (-k)
            want = torch.from_numpy(vals.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            assert np.array_equal(el[0, :16], want), (k, did)
            assert (el[0, 16:] == top).all()
            seen.update(want.tolist())
    assert 0 in seen and 1 in seen and any(2 <= v < 8 for v in seen)     # zero, the smallest subnormal, others


# ------------------------------------------------- sub-formatbook construction
def test_seda_profile_picks_the_most_frequent_dialect_of_each_range(fbk):
    # hand-made metadata: group 0 anchors are rows 0 and 2, group 1 anchor is row 3, row 1 is no anchor
    buckets = range_buckets(fbk)                           # range k -> list of DIDs whose largest magnitude is 8 + k
    d8, d15 = buckets[0], buckets[7]
    assert len(d8) >= 2 and len(d15) >= 3
    e = 130 << 8
    meta = np.array([[d8[1], d8[1], d15[2], d15[0]],
                     [d8[0], d8[0], d8[0], d8[0]],
                     [d8[0], d15[2], d15[1], d15[1]],
                     [d15[1], d15[1], d15[1], d8[1]]], dtype=np.uint16) | e
    counts, sub = O.seda_profile(fbk, meta, np.array([0, -1, 0, 1], dtype=np.int32), 2)
    assert counts.sum() == 12 and counts[0, d8[1]] == 2 and counts[0, d8[0]] == 1 and counts[0, d15[2]] == 2
    assert counts[0, d15[1]] == 2 and counts[0, d15[0]] == 1
    assert sub[0, 0] == d8[1]                              # two selections beat one
    assert sub[0, 7] == min(d15[1], d15[2])                # a tie goes to the lower DID
    assert sub[1, 0] == d8[1] and sub[1, 7] == d15[1]
    for k in range(1, 7):                                  # never selected: the first dialect of the bucket
        assert sub[0, k] == buckets[k][0] and sub[1, k] == buckets[k][0]
    # a formatbook without some ranges: those buckets are marked 255
    small = fbk[[0, 3, 31]]
    _, sub = O.seda_profile(small, np.array([[0, 1, 2, 2]], dtype=np.uint16) | e, np.array([0], dtype=np.int32), 1)
    tops = small[:, 7].astype(int) - 8
    want = np.full(8, 255)
    for d, k in enumerate(tops):
        if want[k] == 255:
            want[k] = d
    assert sub[0].tolist() == want.tolist()


def test_seda_profile_on_a_quantized_tensor_restricts_to_dialects_that_were_in_use(fbk):
    x, comp = synth.mixture_activation(rows=128, cols=1024, seed=36, n_components=4)
    xb = synth.bf16_bits(x)
    c, m = O.quantize(fbk, xb)
    anchors = np.where(np.arange(128) % 4 == 0, comp, -1).astype(np.int32)     # every fourth token is an anchor
    counts, sub = O.seda_profile(fbk, m, anchors, 4)
    for g in range(4):
        rows = np.nonzero(anchors == g)[0]
        assert counts[g].sum() == rows.size * m.shape[1]
        assert np.array_equal(counts[g], np.bincount((m[rows] & 0xFF).ravel(), minlength=32))
        for k in range(8):
            d = int(sub[g, k])
            assert fbk[d, 7] == 8 + k
            same_range = np.nonzero(fbk[:, 7] == 8 + k)[0]
            assert counts[g, d] == counts[g, same_range].max()
    # the constructed tables are valid SeDA inputs: every DID of the restricted pass comes from its row's table
    c2, m2 = O.quantize(fbk, xb, token_group=comp, sub_formatbooks=sub)
    assert ((m2 & 0xFF)[:, :, None] == sub[comp][:, None, :]).any(axis=2).all()


# ------------------------------------------------- LayerNorm producer in front of the quantizer (App. E.2)
def bf16_rne_of_f64(v):
    """float64 -> bf16 bit patterns with ONE rounding to nearest even, by integer arithmetic on the float64 bit
    pattern (normal bf16 range and zero only)."""
    v = np.asarray(v, dtype=np.float64)
    u = v.view(np.uint64)
    sign = (u >> np.uint64(63)).astype(np.uint64)
    ex = ((u >> np.uint64(52)) & np.uint64(0x7FF)).astype(np.int64) - 1023
    man = u & np.uint64((1 << 52) - 1)
    assert ((v == 0) | ((ex >= -126) & (ex <= 127))).all()
    keep = man >> np.uint64(45)                                  # 7 mantissa bits
    rem = man & np.uint64((1 << 45) - 1)
    half = np.uint64(1 << 44)
    up = (rem > half) | ((rem == half) & ((keep & np.uint64(1)) == 1))
    body = ((ex + 127).astype(np.uint64) << np.uint64(7)) + keep + up.astype(np.uint64)   # a carry walks into the exponent
    body = np.where(v == 0, np.uint64(0), body)
    return ((sign << np.uint64(15)) | body).astype(np.uint16)


def test_layernorm_hand_worked_rows():
    # [2,-2,2,-2]: mean 0, biased variance 4, eps 0 -> t = +-1; y = t * gamma + beta
    x = f2b([[2, -2, 2, -2]])
    y, mean, rstd = O.layernorm(x, gamma=[1, 2, 3, 4], beta=[10, 20, 30, 40], eps=0.0)
    assert b2f(y).tolist() == [[11.0, 18.0, 33.0, 36.0]]
    assert mean[0] == 0.0 and rstd[0] == 0.5
    # biased variance: [1,-1] has variance 1, not 2
    y, _, _ = O.layernorm(f2b([[1, -1]]), eps=0.0)
    assert b2f(y).tolist() == [[1.0, -1.0]]
    # eps is added to the variance, inside the root: variance 1, eps 3 -> divide by 2
    y, _, _ = O.layernorm(f2b([[1, -1]]), eps=3.0)
    assert b2f(y).tolist() == [[0.5, -0.5]]
    # the mean is removed: [5, 1] -> mean 3, variance 4 -> +-1
    y, mean, rstd = O.layernorm(f2b([[5, 1]]), eps=0.0)
    assert b2f(y).tolist() == [[1.0, -1.0]] and mean[0] == 3.0 and rstd[0] == 0.5
    # gamma multiplies, beta is added afterwards, each by channel
    y, _, _ = O.layernorm(f2b([[5, 1]]), gamma=[2, 8], beta=[0.5, -0.5], eps=0.0)
    assert b2f(y).tolist() == [[2.5, -8.5]]
    # [1,-1,3,-3]: variance 5; 1/sqrt(5) = 0.4472136 -> bf16 0x3EE5, 3/sqrt(5) = 1.3416408 -> bf16 0x3FAC
    y, _, _ = O.layernorm(f2b([[1, -1, 3, -3]]), eps=0.0)
    assert y.tolist() == [[0x3EE5, 0xBEE5, 0x3FAC, 0xBFAC]]


def test_layernorm_equals_the_library_routine_in_float64_rounded_once():
    # torch's own layer_norm evaluated in float64, then one rounding to bf16 done here by integer arithmetic.
    # Two float64 evaluations of the same value differ by a few 1e-16: a different bf16 only within that of a tie.
    rng = np.random.default_rng(71)
    for rows, cols, mu, sigma in [(64, 96, 0.0, 1.0), (32, 3072, 0.0, 1.0), (16, 1152, 100.0, 1.0), (16, 64, -3.0, 20.0),
                                  (8, 12288, 0.5, 3.0)]:
        xb = f2b(mu + sigma * rng.standard_normal((rows, cols)))
        gamma, beta = synth.layernorm_affine(cols, seed=rows)
        y, mean, rstd = O.layernorm(xb, gamma, beta, eps=1e-6)
        x64 = torch.from_numpy(b2f(xb))
        eps32 = float(np.float32(1e-6))
        ref = torch.nn.functional.layer_norm(x64, (cols,), torch.from_numpy(gamma).double(), torch.from_numpy(beta).double(),
                                             eps32).numpy()
        want = bf16_rne_of_f64(ref)
        diff = np.nonzero(y != want)
        lo, hi = b2f(np.minimum(y, want)[diff]), b2f(np.maximum(y, want)[diff])
        assert (np.abs(ref[diff] - (lo + hi) / 2) <= 1e-13 * np.abs(ref[diff])).all()
        assert diff[0].size <= 2
        # the row statistics, against exactly rounded sums
        for r in (0, rows - 1):
            xs = b2f(xb[r]).tolist()
            m = math.fsum(xs) / cols
            v = math.fsum((t - m) ** 2 for t in xs) / cols
            assert abs(mean[r] - m) <= 1e-13 * max(1.0, abs(m)) and abs(rstd[r] - 1.0 / math.sqrt(v + eps32)) <= 1e-12 * rstd[r]


def test_layernorm_rounding_interval_in_exact_rational_arithmetic():
    # without scale and shift y^2 (var + eps) = (x - mean)^2 exactly; the oracle's bf16 result must be the bf16
    # value whose rounding interval holds the true y -- checked on squares, in rationals, with no square root
    rng = np.random.default_rng(75)
    xb = f2b(rng.standard_normal((6, 12)) * np.array([[1], [3], [0.1], [50], [1], [7]]) + np.array([[0], [1], [0], [-20], [4], [0]]))
    eps = Fraction(float(np.float32(1e-3)))
    y, _, _ = O.layernorm(xb, eps=float(np.float32(1e-3)))
    for r in range(6):
        xs = [exact(int(b)) for b in xb[r]]
        mean = sum(xs) / 12
        var = sum((t - mean) ** 2 for t in xs) / 12
        for c in range(12):
            d = xs[c] - mean
            yb = int(y[r, c])
            assert (yb >> 15) == (1 if d < 0 else 0)
            mag = yb & 0x7FFF
            lo = (exact(mag - 1) + exact(mag)) / 2 if mag else Fraction(0)     # neighbours' midpoints
            hi = (exact(mag) + exact(mag + 1)) / 2
            t2 = d * d / (var + eps)                                           # the true y, squared
            assert lo * lo <= t2 <= hi * hi


def test_layernorm_invariants():
    rng = np.random.default_rng(72)
    xb = f2b(rng.standard_normal((8, 256)))
    gamma, beta = synth.layernorm_affine(256, seed=3)
    y, mean, rstd = O.layernorm(xb, gamma, beta, eps=0.0)
    # scaling a row by a power of two changes nothing when eps = 0 (every step scales exactly)
    y4, mean4, rstd4 = O.layernorm(f2b(b2f(xb) * 4.0), gamma, beta, eps=0.0)
    assert np.array_equal(y, y4) and np.array_equal(rstd4 * 4, rstd) and np.array_equal(mean4, 4 * mean)
    # rows are independent, and a row stride changes nothing
    wide = np.zeros((8, 300), dtype=np.uint16)
    wide[:, :256] = xb
    wide[:, 256:] = 0x7FC0
    ys, _, _ = O.layernorm(wide[:, :256], gamma, beta, eps=0.0)
    assert np.array_equal(ys, y)
    y1, _, _ = O.layernorm(xb[3:4], gamma, beta, eps=0.0)
    assert np.array_equal(y1[0], y[3])
    # negating the input negates the normalized value: with beta = 0 the output changes sign only
    yn, _, _ = O.layernorm(xb ^ 0x8000, gamma, None, eps=0.0)
    yp, _, _ = O.layernorm(xb, gamma, None, eps=0.0)
    assert np.array_equal(yn ^ 0x8000, yp)
    # shifting a row by a constant changes nothing (the shift is chosen so that x + 8 is exact in bf16)
    xq = f2b(np.round(b2f(xb) * 8) / 8)
    ya, _, _ = O.layernorm(xq, gamma, beta, eps=1e-6)
    yb, _, _ = O.layernorm(f2b(b2f(xq) + 8.0), gamma, beta, eps=1e-6)
    assert np.array_equal(b2f(f2b(b2f(xq) + 8.0)), b2f(xq) + 8.0) and (ya == yb).mean() > 0.999
    # a constant row has variance 0 and every x - mean is 0: y is exactly beta (rounded to bf16), whatever eps
    for value, cols in ((1.5, 256), (-1000.0, 3072), (3.0e-5, 96)):
        g, b = synth.layernorm_affine(cols, seed=5)
        const = f2b(np.full((1, cols), value))
        yc, mc, rc = O.layernorm(const, g, b, eps=1e-6)
        assert np.array_equal(yc[0], f2b(b)) and mc[0] == float(b2f(const)[0, 0])
        assert abs(rc[0] - 1.0 / math.sqrt(float(np.float32(1e-6)))) < 1e-9
    # a zero row with gamma only: exactly zero
    yz, mz, rz = O.layernorm(np.zeros((1, 256), dtype=np.uint16), gamma, None, eps=1e-6)
    assert not (yz & 0x7FFF).any() and mz[0] == 0.0
    # without scale and shift the normalized row has mean 0 and second moment var / (var + eps), up to bf16 rounding
    yn, _, _ = O.layernorm(xb, eps=1e-6)
    assert np.abs(b2f(yn).mean(axis=1)).max() < 2e-3 and np.abs((b2f(yn) ** 2).mean(axis=1) - 1.0).max() < 5e-3


def test_layernorm_rows_with_nan_or_inf_become_canonical_nan():
    rng = np.random.default_rng(73)
    xb = f2b(rng.standard_normal((4, 64)))
    clean, _, _ = O.layernorm(xb)
    xb[1, 5] = 0xFFC1          # a negative NaN with a payload
    xb[2, 60] = 0x7F80         # +Inf
    y, _, _ = O.layernorm(xb)
    assert (y[1] == 0x7FC0).all() and (y[2] == 0x7FC0).all()
    assert np.array_equal(y[0], clean[0]) and np.array_equal(y[3], clean[3])


def test_layernorm_then_quantize_sees_unit_scale_blocks(fbk):
    # after LayerNorm without affine a row has unit variance: the block maxima of a Gaussian row (32 draws) sit
    # in [1, 4) for nearly every block, whatever the scale of the input was
    rng = np.random.default_rng(74)
    xb = f2b(1e4 * rng.standard_normal((4, 3072)))
    y, _, _ = O.layernorm(xb)
    _, m = O.quantize(fbk, y)
    e = (m >> 8).astype(int) - 127
    assert np.isin(e, (0, 1)).mean() > 0.98 and e.max() <= 2 and e.min() >= -1
    _, m_raw = O.quantize(fbk, xb)
    assert ((m_raw >> 8).astype(int) - 127).min() >= 12


# ------------------------------------------------- GeLU producer in front of the quantizer (App. E.2)
ALL_BF16 = np.arange(65536, dtype=np.uint16)


def _bf16_of_f64(v):
    """float64 -> bf16 bits through torch (float64 -> float32 -> bf16; a double rounding that matters only
    within 2^-29 of a tie, which no value below hits)."""
    return torch.from_numpy(np.asarray(v, dtype=np.float64)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


@pytest.mark.parametrize("approximate", [0, 1])
def test_gelu_equals_the_library_routine_on_every_bf16_value_where_that_is_accurate(approximate):
    y = O.gelu(ALL_BF16, approximate)
    x = b2f(ALL_BF16)
    ref = torch.nn.functional.gelu(torch.from_numpy(x), approximate="tanh" if approximate else "none").numpy()
    # 0.5 x (1 + erf) / 0.5 x (1 + tanh) cancel for x << 0: the library's float64 result is good to the last
    # bf16 bit down to about -5; the tail is pinned by the next test
    ok = np.isfinite(x) & (x > -5.0)
    assert np.array_equal(y[ok], _bf16_of_f64(ref[ok]))
    # specials: NaN -> canonical quiet NaN, +Inf -> +Inf, -Inf -> -0 (the limit), signed zeros kept
    nan = (ALL_BF16 & 0x7FFF) > 0x7F80
    assert (y[nan] == 0x7FC0).all() and y[0x7F80] == 0x7F80 and y[0xFF80] == 0x8000
    assert y[0x0000] == 0x0000 and y[0x8000] == 0x8000


def test_gelu_negative_tail_against_bounds_and_the_other_closed_form():
    x = b2f(ALL_BF16)
    neg = np.isfinite(x) & (x <= -5.0)
    t = -x[neg]
    # exact form: x Phi(x); Mills-ratio bounds  phi(t) t / (t^2 + 1) < Phi(-t) < phi(t) / t
    with np.errstate(under="ignore"):
        phi = np.exp(-0.5 * t * t) / math.sqrt(2.0 * math.pi)
        lo = t * phi * t / (t * t + 1.0)        # |y| lower bound
        hi = phi                                 # |y| upper bound (t * phi / t)
    y = -b2f(O.gelu(ALL_BF16[neg], 0))
    step = 1.0 + 2.0 ** -7
    tiny = 2.0 ** -133                           # the smallest bf16 step near zero
    assert (y <= hi * step + tiny).all() and (y >= lo / step - tiny).all()
    # tanh form: 0.5 x (1 + tanh u) = x e^{2u} / (1 + e^{2u}), accurate for u << 0
    u = math.sqrt(2.0 / math.pi) * (x[neg] + 0.044715 * x[neg] ** 3)
    with np.errstate(under="ignore"):
        e2 = np.exp(2.0 * u)
        ref = x[neg] * e2 / (1.0 + e2)
    assert np.array_equal(O.gelu(ALL_BF16[neg], 1), _bf16_of_f64(ref) | np.uint16(0x8000))


@pytest.mark.parametrize("approximate", [0, 1])
def test_gelu_shape_of_the_function(approximate):
    y = b2f(O.gelu(ALL_BF16, approximate))
    x = b2f(ALL_BF16)
    fin = np.isfinite(x)
    pos = fin & (x >= 0)
    # identity from x = 8 upwards (1 - Phi(8) is far below half a bf16 step), x / 2 near zero
    big = pos & (x >= 8.0)
    assert np.array_equal(O.gelu(ALL_BF16[big], approximate), ALL_BF16[big])
    small = fin & (np.abs(x) < 2.0 ** -12) & (np.abs(x) >= 2.0 ** -120)
    assert np.array_equal(y[small], x[small] / 2)
    # GeLU(x) - GeLU(-x) = x, up to the two roundings
    a = ALL_BF16[pos]
    d = y[a] - y[a | 0x8000]
    assert (np.abs(d - x[pos]) <= 2.0 ** -7 * x[pos] + 2.0 ** -133).all()
    # increasing on x >= 0, bounded below by about -0.17 (attained near x = -0.75), never positive for x < 0
    assert (np.diff(y[pos][np.argsort(x[pos], kind="stable")]) >= 0).all()
    negv = y[fin & (x < 0)]
    assert negv.max() <= 0 and abs(negv.min() + 0.17) < 0.005
    assert abs(x[fin & (x < 0)][np.argmin(negv)] + 0.75) < 0.1      # (flat at bf16 resolution around the minimum)
    # one worked value: GeLU(1) = 0.841345 (exact form), 0.841192 (tanh form) -> both bf16 0x3F57 = 0.83984375
    assert O.gelu(f2b([1.0]), approximate)[0] == 0x3F57
    # ... and one where the two forms differ: GeLU(3) = 2.995950 -> 0x4040 (3.0); tanh form 2.996363 -> 0x4040
    assert O.gelu(f2b([-2.0]), 0)[0] == f2b([-0.04550026])[0] and O.gelu(f2b([-2.0]), 1)[0] == f2b([-0.04540231])[0]


# ------------------------------------------------- attention-guided salient tokens (Sec. 3.3, App. F)
def test_attention_scores_hand_worked_and_brute_force():
    # two tokens, two channels: Q = [[1, 0], [0, 2]], K = [[1, 1], [-1, 0.5]]; QK^T = [[1, -1], [2, 1]]
    q = f2b([[[1, 0], [0, 2]]])
    k = f2b([[[1, 1], [-1, 0.5]]])
    assert O.attention_scores(q, k, "abs").tolist() == [[1.0, 1.5]]          # (|1| + |-1|) / 2, (2 + 1) / 2
    assert O.attention_scores(q, k, "relu").tolist() == [[0.5, 1.5]]         # (1 + 0) / 2, (2 + 1) / 2
    # plain loops in exact rational arithmetic on a small random case
    rng = np.random.default_rng(81)
    qb, kb = f2b(rng.standard_normal((3, 5, 8))), f2b(rng.standard_normal((3, 5, 8)))
    for mode in ("abs", "relu"):
        got = O.attention_scores(qb, kb, mode)
        for g in range(3):
            for i in range(5):
                acc = Fraction(0)
                for j in range(5):
                    dot = sum(exact(int(a)) * exact(int(b)) for a, b in zip(qb[g, i], kb[g, j]))
                    acc += abs(dot) if mode == "abs" else max(dot, Fraction(0))
                assert abs(got[g, i] - float(acc / 5)) <= 1e-12 * max(1.0, float(acc))


def test_attention_scores_against_the_library_contraction_and_invariants():
    rng = np.random.default_rng(82)
    qb, kb = f2b(rng.standard_normal((4, 96, 64))), f2b(rng.standard_normal((4, 96, 64)))
    q, k = torch.from_numpy(b2f(qb)), torch.from_numpy(b2f(kb))
    s = torch.einsum("gqc,gkc->gqk", q, k)
    assert np.allclose(O.attention_scores(qb, kb, "abs"), s.abs().mean(dim=2).numpy(), rtol=1e-12, atol=0)
    assert np.allclose(O.attention_scores(qb, kb, "relu"), s.clamp(min=0).mean(dim=2).numpy(), rtol=1e-12, atol=0)
    # |.| does not see the sign of K; relu(s) - relu(-s) = s and relu(s) + relu(-s) = |s|
    a = O.attention_scores(qb, kb, "abs")
    assert np.array_equal(a, O.attention_scores(qb, kb ^ 0x8000, "abs"))
    rp, rn = O.attention_scores(qb, kb, "relu"), O.attention_scores(qb, kb ^ 0x8000, "relu")
    assert np.allclose(rp + rn, a, rtol=1e-12) and np.allclose(rp - rn, s.mean(dim=2).numpy(), rtol=1e-9, atol=1e-12)
    # groups are independent, keys may come in any order, scaling Q by 2 doubles the score
    assert np.array_equal(O.attention_scores(qb[1:2], kb[1:2], "abs")[0], a[1])
    assert np.allclose(O.attention_scores(qb, kb[:, ::-1], "abs"), a, rtol=1e-12)
    assert np.array_equal(O.attention_scores(f2b(b2f(qb) * 2), kb, "abs"), 2 * a)


def test_salient_token_selection_per_tile():
    # 4 x 4 grid, 2 x 2 tiles, two heads: hand-made scores
    s = np.zeros((1, 2, 16))
    s[0, 0, 5] = 1; s[0, 1, 5] = 1            # tile (0,0): token 5, mean 1
    s[0, 0, 2] = 3                            # tile (0,1): token 2, mean 1.5 (one head only)
    s[0, 1, 10] = 2.5; s[0, :, 15] = np.nan   # tile (1,1): token 10; a NaN never wins.  tile (1,0): all equal -> 8
    assert O.select_salient_tokens(s, 4, 4, 2, 2).tolist() == [[2, 5, 8, 10]]
    # tiles that are not square: 4 x 6 grid, tiles 2 high and 3 wide; the best of tile (0,1) = columns 3-5 of rows 0-1
    s2 = np.zeros((1, 1, 24))
    s2[0, 0, 2 * 6 + 1] = 5          # row 2, col 1 -> tile (1,0)
    s2[0, 0, 1 * 6 + 4] = 7          # row 1, col 4 -> tile (0,1)
    s2[0, 0, 3 * 6 + 5] = 1          # row 3, col 5 -> tile (1,1)
    assert O.select_salient_tokens(s2, 4, 6, 2, 3).tolist() == [[0, 10, 13, 23]]
    # ragged tiles, several frames: one token per tile, inside its tile, with the tile's largest mean
    rng = np.random.default_rng(83)
    sc = rng.random((3, 5, 7 * 10)).astype(np.float32)
    out = O.select_salient_tokens(sc, 7, 10, 4, 4)
    assert out.shape == (3, 2 * 3) and (np.diff(out, axis=1) > 0).all()
    mean = sc.astype(np.float64).mean(axis=1)
    for f in range(3):
        seen = set()
        for row in out[f]:
            t = int(row) - f * 70
            y, x = divmod(t, 10)
            tile = (y // 4, x // 4)
            assert tile not in seen
            seen.add(tile)
            ys, xs = range(tile[0] * 4, min(7, tile[0] * 4 + 4)), range(tile[1] * 4, min(10, tile[1] * 4 + 4))
            assert mean[f, t] == max(mean[f, yy * 10 + xx] for yy in ys for xx in xs)
        assert len(seen) == 6


def test_seda_assignment_marks_the_window_tokens_an_anchor_attends_to():
    # one frame, one head, 4 x 4 grid, 2 x 2 tiles, 2 channels; anchors at tokens 5 (tile 0) and 10 (tile 3); window 3
    q = np.zeros((1, 1, 16, 2), dtype=np.float32)
    k = np.zeros((1, 1, 16, 2), dtype=np.float32)
    q[0, 0, 5] = [1, 0]; q[0, 0, 10] = [0, 1]
    k[0, 0, :, 0] = [0, 9, 0, 0,  2, 0, 7, 0,  0, 6, 0, 0,  0, 0, 0, 0]      # what anchor 5 sees
    k[0, 0, :, 1] = [0, 0, 0, 0,  0, 8, 6.5, 0,  0, 0, 0, 9,  0, 0, 9, 5]    # what anchor 10 sees
    tg, ag, sc = O.seda_assign(f2b(q), f2b(k), [5, 10], 1, 4, 4, tile_h=2, tile_w=2, window=3, threshold=5.0)
    # anchor 5 (row 1, col 1) sees tokens 0-2, 4-6, 8-10: above 5 are 1 (9), 6 (7), 9 (6)
    # anchor 10 (row 2, col 2) sees 5-7, 9-11, 13-15: above 5 are 5 (8), 6 (6.5), 11 (9), 14 (9); 15 (5) is not above
    want = np.full(16, -1)
    want[[1, 9]] = 0
    want[[6, 11, 14]] = 3          # token 6: both anchors -> the later tile
    want[5] = 0; want[10] = 3      # anchors keep their own group (anchor 10 marked token 5, but 5 is an anchor)
    assert tg.tolist() == want.tolist()
    assert ag.tolist() == [-1] * 5 + [0] + [-1] * 4 + [3] + [-1] * 5
    assert sc[0].tolist() == [0, 9, 0, 2, 0, 7, 0, 6, 0] and sc[1, 8] == 5.0
    # the order of the list does not matter, and an entry outside the tensor does nothing
    tg2, ag2, sc2 = O.seda_assign(f2b(q), f2b(k), [-1, 10, 16, 5], 1, 4, 4, tile_h=2, tile_w=2, window=3, threshold=5.0)
    assert np.array_equal(tg2, tg) and np.array_equal(ag2, ag) and np.isnan(sc2[0]).all() and np.isnan(sc2[2]).all()
    assert np.array_equal(sc2[3], sc[0])
    # a window clipped by the frame edge, two heads averaged, negative scores never mark
    q2 = np.zeros((1, 2, 16, 2), dtype=np.float32); k2 = np.zeros((1, 2, 16, 2), dtype=np.float32)
    q2[0, :, 0] = [1, 0]
    k2[0, 0, :, 0] = [0, 12, 0, 0, -20, 4, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0]
    k2[0, 1, :, 0] = [0, 0, 0, 0, -20, 8, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0]
    tg, _, sc = O.seda_assign(f2b(q2), f2b(k2), [0], 1, 4, 4, tile_h=2, tile_w=2, window=3, threshold=5.0)
    assert tg.tolist() == [0, 0, -1, -1, -1, 0] + [-1] * 10           # token 1: (12 + 0) / 2 = 6, token 5: 6, token 4: -20
    assert np.isnan(sc[0, :3]).all() and np.isnan(sc[0, 3]) and sc[0, 5] == 6.0


def test_seda_groups_are_tiles_shared_by_the_frames():
    # Sec. 3.4 step 1: the N per-frame candidates of ONE tile share a sub-formatbook.  Two frames of an 8 x 8 grid
    # with 4 x 4 tiles; in frame 0 tile (0,0)'s candidate sits in grid row 3 (token 24) and tile (0,1)'s in grid row 0
    # (token 4), so the ascending list of frame 0 starts with the candidate of tile (0,1), that of frame 1 with the
    # candidate of tile (0,0): the group must follow the tile, not the position in the list.
    scores = np.zeros((2, 1, 64))
    scores[0, 0, [24, 4, 33, 63]] = 1.0          # frame 0: tiles (0,0) (0,1) (1,0) (1,1)
    scores[1, 0, [0, 7, 32, 39]] = 1.0           # frame 1
    picks = O.select_salient_tokens(scores, 8, 8, 4, 4)
    assert picks.tolist() == [[4, 24, 33, 63], [64, 71, 96, 103]]
    q = np.zeros((2, 1, 64, 8), dtype=np.uint16)
    tg, ag, _ = O.seda_assign(q, q, picks.ravel(), 2, 8, 8, tile_h=4, tile_w=4, window=5, threshold=1.0)
    assert [int(ag[r]) for r in (24, 4, 33, 63)] == [0, 1, 2, 3]
    assert [int(ag[64 + t]) for t in (0, 7, 32, 39)] == [0, 1, 2, 3]
    assert (ag >= 0).sum() == 8 and np.array_equal(tg, ag)      # all scores are 0: nothing but the anchors is marked
    # the profile then pools the anchors of one tile: group 0 = rows 24 and 64
    meta = np.zeros((128, 1), dtype=np.uint16)
    meta[24, 0] = 3; meta[64, 0] = 3; meta[4, 0] = 5; meta[71, 0] = 5
    counts, _ = O.seda_profile(DEFAULT_FORMATBOOK, meta, ag, 4)
    assert counts[0, 3] == 2 and counts[1, 5] == 2 and counts[0].sum() == 2


def test_seda_main_anchor_and_frame_pruning_hand_worked():
    # Sec. 3.4 step 2.  Three frames of a 2 x 2 grid, one 2 x 2 tile, one channel.  Candidates: frame 0 token 1,
    # frame 1 token 2, frame 2 token 1.  Temporal mean scores of the candidates: 2, 5, 3 -> main anchor = frame 1's
    # (row 6, position 2).  Raw temporal scores from the main anchor: Qt[2][f = 1] = 2 times Kt[2][f] = 1, .5, 4
    # -> 2, 1, 8; threshold 3: frame 0 is pruned, frame 2 stays, the main anchor's own frame stays although 1 < 3.
    ts = np.zeros((4, 1, 3))
    ts[1, 0, 0] = 2.0; ts[2, 0, 1] = 5.0; ts[1, 0, 2] = 3.0
    qt = np.zeros((4, 1, 3, 1), dtype=np.float32); kt = np.zeros((4, 1, 3, 1), dtype=np.float32)
    qt[2, 0, 1, 0] = 2.0
    kt[2, 0, :, 0] = [1.0, 0.5, 4.0]
    cand = [[1], [6], [9]]
    main, kept, ps = O.seda_main_anchor(ts, f2b(qt), f2b(kt), cand, 2, 2, 2, 2, prune_threshold=3.0)
    assert main.tolist() == [6] and kept.tolist() == [[-1], [6], [9]] and ps[:, 0].tolist() == [2.0, 1.0, 8.0]
    # on a tie the earliest frame is the main anchor; a NaN score never wins; an entry outside its frame is no
    # candidate; heads are averaged (scores 2 and 6 -> 4 > 3.5)
    ts2 = np.zeros((4, 2, 3))
    ts2[1, :, 0] = [4.0, 6.0]; ts2[2, :, 1] = [np.nan, 9.0]; ts2[1, :, 2] = [5.0, 5.0]
    qt2 = np.zeros((4, 2, 3, 1), dtype=np.float32); kt2 = np.zeros((4, 2, 3, 1), dtype=np.float32)
    qt2[1, :, 0, 0] = [1.0, 2.0]
    kt2[1, :, 2, 0] = [2.0, 3.0]
    main, kept, ps = O.seda_main_anchor(ts2, f2b(qt2), f2b(kt2), [[1, 3], [6, 0], [9, 30]], 2, 2, 2, 2, prune_threshold=3.5)
    assert main.tolist() == [1]                      # 5 = 5: frame 0 before frame 2; frame 1's mean is NaN
    assert ps[2, 0] == 4.0 and ps[1, 0] == 0.0       # (1*2 + 2*3) / 2
    assert kept.tolist() == [[1, -1], [-1, -1], [9, -1]]
    # two tiles side by side: each tile has its own main anchor
    ts3 = np.zeros((8, 1, 2))
    ts3[0, 0, 0] = 1.0; ts3[5, 0, 1] = 2.0           # tile 0: frame 0 token 0, frame 1 token 5 -> main = row 8 + 5
    ts3[2, 0, 0] = 3.0; ts3[7, 0, 1] = 1.0           # tile 1: frame 0 token 2, frame 1 token 7 -> main = row 2
    z = np.zeros((8, 1, 2, 1), dtype=np.uint16)
    main, kept, _ = O.seda_main_anchor(ts3, z, z, [[0, 2], [13, 15]], 2, 4, 2, 2, prune_threshold=-1.0)
    assert main.tolist() == [13, 2] and kept.tolist() == [[0, 2], [13, 15]]
    main, kept, _ = O.seda_main_anchor(ts3, z, z, [[0, 2], [13, 15]], 2, 4, 2, 2, prune_threshold=0.0)
    assert kept.tolist() == [[-1, 2], [13, -1]]      # a score of 0 does not exceed 0


def test_seda_3d_main_anchor_and_cuboid_window_hand_worked():
    # Sec. 3.4, 3D attention: two frames of a 2 x 4 grid, 2 x 2 tiles -> two tiles of 2 x 2 x 2 tokens.
    sc = np.zeros((2, 16))
    sc[0, 13] = 1.0; sc[1, 13] = 2.0                 # tile 0: frame 1, token 5 (head mean 1.5)
    sc[0, 0] = 1.0; sc[1, 0] = 1.5                   # ... beats frame 0, token 0 (1.25)
    sc[:, 2] = 0.75; sc[:, 10] = 0.75                # tile 1: a tie between row 2 and row 8 + 2 -> the lower row
    sc[0, 7] = np.nan                                # a NaN never wins
    anchors = O.seda_main_anchor_3d(sc, 2, 2, 4, 2, 2)
    assert anchors.tolist() == [13, 2]
    # cuboid window 3 x 3 x 3 around row 13 = (frame 1, row 1, col 1): frames 0-1 (clipped), rows 0-1, cols 0-2
    q = np.zeros((1, 16, 1), dtype=np.float32); k = np.zeros((1, 16, 1), dtype=np.float32)
    q[0, 13, 0] = 1.0; q[0, 2, 0] = -1.0
    k[0, :, 0] = [6, 0, 7, 9,  0, 5, -8, 0,   0, 7, 0, 9,  3, 0, 8, -9]
    tg, ag, s = O.seda_assign(f2b(q), f2b(k), anchors, 2, 2, 4, tile_h=2, tile_w=2, window=3, window_t=3, threshold=5.0,
                              joint=True)
    # anchor 13 (group 0) sees rows {0,1,2,4,5,6} and {8,9,10,12,13,14}: above 5 are 0 (6), 2 (7), 9 (7), 14 (8)
    # anchor 2 = (frame 0, row 0, col 2) (group 1) sees cols 1-3 of both frames with scores -k: above 5 are 6 (8), 15 (9)
    want = np.full(16, -1)
    want[[0, 9, 14]] = 0
    want[[6, 15]] = 1
    want[13] = 0; want[2] = 1                        # row 2 was marked by anchor 13 but is an anchor itself
    assert tg.tolist() == want.tolist()
    assert ag.tolist() == [-1, -1, 1] + [-1] * 10 + [0, -1, -1]
    # slots: frame offset major; the first frame offset (-1 from frame 1 = frame 0) holds rows 0-2, 4-6
    assert s.shape == (2, 27) and s[0, :6].tolist() == [6, 0, 7, 0, 5, -8]
    assert np.isnan(s[0, 6:9]).all() and np.isnan(s[0, 18:]).all() and s[0, 9:15].tolist() == [0, 7, 0, 3, 0, 8]
    # with window_t = 1 the anchors only see their own frame
    tg1, _, _ = O.seda_assign(f2b(q), f2b(k), anchors, 2, 2, 4, tile_h=2, tile_w=2, window=3, window_t=1, threshold=5.0,
                              joint=True)
    want1 = np.full(16, -1)
    want1[[9, 14]] = 0; want1[6] = 1; want1[13] = 0; want1[2] = 1
    assert tg1.tolist() == want1.tolist()


def test_seda_tiles_that_are_not_square_hand_worked():
    # A 4 x 6 grid cut into tiles of 2 rows x 3 columns: 2 x 2 tiles, numbered row-major
    #   tokens  0  1  2 |  3  4  5      tile 0 | tile 1
    #           6  7  8 |  9 10 11
    #          ---------+---------
    #          12 13 14 | 15 16 17      tile 2 | tile 3
    #          18 19 20 | 21 22 23
    # (tile_h and tile_w exchanged, or the tile grid transposed, would give other numbers for tokens 8, 9, 12.)
    q = np.zeros((1, 1, 24, 1), dtype=np.uint16)
    anchors = [8, 9, 12, 23]
    _, ag, _ = O.seda_assign(q, q, anchors, 1, 4, 6, tile_h=2, tile_w=3, window=3, threshold=1.0)
    assert [int(ag[t]) for t in anchors] == [0, 1, 2, 3]
    # the per-tile choice and the 3D main anchor use the same tiles: one frame, one head, the best token of
    # each tile planted at 8, 9, 12, 23; a 4 x 9 grid with the same tiles has 2 x 3 tiles, the last row of
    # tiles being numbers 3, 4, 5
    sc = np.zeros((1, 24)); sc[0, anchors] = 1.0
    assert O.seda_main_anchor_3d(sc, 1, 4, 6, 2, 3).tolist() == anchors
    assert O.select_salient_tokens(sc.reshape(1, 1, 24), 4, 6, 2, 3).tolist() == [anchors]
    sc = np.zeros((1, 36)); sc[0, [2, 12, 8, 18, 31, 26]] = 1.0
    assert O.seda_main_anchor_3d(sc, 1, 4, 9, 2, 3).tolist() == [2, 12, 8, 18, 31, 26]
    # step 2 finds a candidate's tile the same way: one frame, candidates 8 and 12 -> tiles 0 and 2
    ts = np.ones((24, 1, 1)); z = np.zeros((24, 1, 1, 1), dtype=np.uint16)
    main, kept, _ = O.seda_main_anchor(ts, z, z, [[8, 12]], 4, 6, 2, 3, prune_threshold=0.0)
    assert main.tolist() == [8, -1, 12, -1] and kept.tolist() == [[8, 12]]
