"""Pins for the oracle's other MX element formats (E4M3, E5M2, E2M3, E3M2; Sec. 1, footnote).

The paper gives no number for these formats, so nothing here is a value it prints.  What is pinned is
the reading stated in the oracle (each rule with the element format's own largest value V and top-binade
half-step h in place of E2M1's 6 and 1) against things that do not depend on the oracle: the element
formats as the OCP MX specification defines them and as a library implements the two FP8 ones (torch's
float8 dtypes on the CPU), exact rational arithmetic written out here, the intervals each rule must map
the block maximum into, and the E2M1 functions, which the general ones must reproduce.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2603_08713_amd import synth

FORMATS = ["e4m3", "e5m2", "e2m3", "e3m2"]
# (exponent bits, mantissa bits, bias, largest finite value, smallest subnormal) per the OCP MX specification
SPEC = {
    "e2m1": (2, 1, 1, Fraction(6), Fraction(1, 2)),
    "e4m3": (4, 3, 7, Fraction(448), Fraction(1, 512)),
    "e5m2": (5, 2, 15, Fraction(57344), Fraction(1, 65536)),
    "e2m3": (2, 3, 1, Fraction(15, 2), Fraction(1, 8)),
    "e3m2": (3, 2, 3, Fraction(28), Fraction(1, 16)),
}
TORCH_FP8 = {"e4m3": torch.float8_e4m3fn, "e5m2": torch.float8_e5m2}


def bf16_frac(h: int) -> Fraction:
    sign = -1 if h & 0x8000 else 1
    e, m = (h >> 7) & 0xFF, h & 0x7F
    if e == 0:
        return sign * Fraction(m, 128) * Fraction(2) ** (-126)
    return sign * (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)


def grid(fmt):
    """All finite magnitudes of the format, ascending, built from the specification's definition."""
    eb, mb, bias, vmax, _ = SPEC[fmt]
    vals = []
    for c in range(1 << (eb + mb)):
        e, m = c >> mb, c & ((1 << mb) - 1)
        v = Fraction(m, 1 << mb) * Fraction(2) ** (1 - bias) if e == 0 else (1 + Fraction(m, 1 << mb)) * Fraction(2) ** (e - bias)
        if v <= vmax:
            vals.append(v)
    assert vals == sorted(vals) and vals[-1] == vmax
    return vals


def nearest_code(vals, y: Fraction) -> int:
    """Index of the nearest grid value, ties to the even index, saturating (exact)."""
    if y >= vals[-1]:
        return len(vals) - 1
    return min(range(len(vals)), key=lambda c: (abs(y - vals[c]), c & 1))


def half_step_top(fmt) -> Fraction:
    _, mb, _, vmax, _ = SPEC[fmt]
    emax = max(e for e in range(-20, 20) if Fraction(2) ** e <= vmax)
    return Fraction(2) ** (emax - mb - 1)


# ------------------------------------------------------------------------------------------------
# the element formats
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fmt", FORMATS + ["e2m1"])
def test_elem_decode_matches_the_specification(oracle, fmt):
    eb, mb, _, vmax, vmin = SPEC[fmt]
    vals = grid(fmt)
    assert oracle.elem_bits(fmt) == 1 + eb + mb
    assert Fraction(oracle.elem_max(fmt)) == vmax
    assert Fraction(oracle.elem_decode(fmt, 1)) == vmin
    sign = 1 << (eb + mb)
    for c, v in enumerate(vals):
        assert Fraction(oracle.elem_decode(fmt, c)) == v
        assert Fraction(oracle.elem_decode(fmt, c | sign)) == -v
    # codes past the largest finite one (E4M3's NaN, E5M2's Inf / NaN) are not numbers
    for c in range(len(vals), sign):
        assert np.isnan(oracle.elem_decode(fmt, c))
    assert len(vals) == {"e2m1": 8, "e4m3": 127, "e5m2": 124, "e2m3": 32, "e3m2": 32}[fmt]


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2"])
def test_fp8_decode_and_rounding_match_a_library(oracle, fmt):
    dt = TORCH_FP8[fmt]
    lib_vals = torch.arange(256, dtype=torch.uint8).view(dt).to(torch.float64).numpy()
    for c in range(256):
        o = oracle.elem_decode(fmt, c)
        if np.isfinite(lib_vals[c]):
            assert o == lib_vals[c], c
        else:
            assert np.isnan(o), c
    # rounding of in-range values (the library does not saturate, so stay at or below the largest value):
    # random magnitudes over all binades, every grid point, every midpoint and its neighbours
    rng = np.random.default_rng(1)
    vmax = float(SPEC[fmt][3])
    vals = [float(v) for v in grid(fmt)]
    mids = [(a + b) / 2 for a, b in zip(vals[:-1], vals[1:])]
    y = np.concatenate([np.exp2(rng.uniform(-20, np.log2(vmax), 20000)), vals, mids,
                        np.nextafter(np.float32(mids), np.float32(0)), np.nextafter(np.float32(mids), np.float32(1e9))])
    y = np.minimum(y.astype(np.float32), np.float32(vmax))
    want = torch.from_numpy(y).to(dt).view(torch.uint8).numpy()
    got = np.array([oracle.elem_nearest(fmt, float(v)) for v in y], np.uint8)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("fmt", FORMATS + ["e2m1"])
def test_elem_nearest_against_exact_search(oracle, fmt):
    vals = grid(fmt)
    rng = np.random.default_rng(2)
    ys = [Fraction(float(v)) for v in np.exp2(rng.uniform(-12, float(np.log2(float(vals[-1]))) + 1.5, 3000))]
    ys += vals + [(a + b) / 2 for a, b in zip(vals[:-1], vals[1:])]
    ys += [vals[-1] + Fraction(1, 1024), vals[-1] * 3, Fraction(0)]
    for y in ys:
        assert oracle.elem_nearest(fmt, float(y)) == nearest_code(vals, y), (fmt, y)
    if fmt == "e2m1":
        for y in ys:
            assert oracle.elem_nearest(fmt, float(y)) == oracle.e2m1_nearest(float(y))


# ------------------------------------------------------------------------------------------------
# the scale rules and the MBS word with the format's own constants
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fmt", FORMATS + ["e2m1"])
def test_elem_scale_rule_intervals_all_bf16(oracle, fmt):
    _, _, _, V, _ = SPEC[fmt]
    h = half_step_top(fmt)
    top = max(Fraction(2) ** e for e in range(-20, 20) if Fraction(2) ** e <= V)
    for hbits in range(0x0080, 0x7F80, 7):  # positive normal bf16
        a = bf16_frac(hbits)
        for rule, lo, hi, lo_open in (("floor", V / 2, V, True), ("oas", (V + h) / 2, V + h, True),
                                     ("ocp", top, 2 * top, False)):
            s = oracle.elem_scale_exponent(fmt, float(a), rule)
            y = a * Fraction(2) ** s
            assert (lo < y if lo_open else lo <= y) and (y <= hi if lo_open else y < hi), (fmt, rule, hbits, y)
    if fmt == "e2m1":
        for hbits in range(0x0080, 0x7F80, 5):
            a = float(bf16_frac(hbits))
            for rule in ("floor", "oas", "ocp"):
                assert oracle.elem_scale_exponent(fmt, a, rule) == oracle.scale_exponent(a, rule)


@pytest.mark.parametrize("fmt", FORMATS)
def test_elem_oas_trades_no_error_for_its_wider_range(oracle, fmt):
    """What the reading rests on: a block maximum that OAS lets overflow, (V, V + h], is stored as V with an
    error of at most h, no more than rounding costs inside the top binade; the doubled scale halves the error
    of every other element of the block."""
    _, _, _, V, _ = SPEC[fmt]
    h = half_step_top(fmt)
    vals = grid(fmt)
    assert vals[-1] - vals[-2] == 2 * h
    for y in (V + h, V + h / 2, V + h / 1024):
        assert V - Fraction(oracle.elem_decode(fmt, oracle.elem_nearest(fmt, float(y)))) + y - V <= h


@pytest.mark.parametrize("fmt", FORMATS + ["e2m1"])
def test_elem_mbs_static_maps_macro_max_to_v(oracle, fmt):
    _, _, _, V, _ = SPEC[fmt]
    for hbits in list(range(0x0001, 0x7F80, 11)) + [0x0001, 0x007F, 0x0080, 0x7F7F]:
        a = bf16_frac(hbits)
        m8 = oracle.elem_mbs_static_m8(fmt, float(a))
        # exact: the 8 leading mantissa bits of V / a
        q = V / a
        while q >= 2:
            q /= 2
        while q < 1:
            q *= 2
        assert m8 == int((q - 1) * 256), (fmt, hbits)
        if fmt == "e2m1":
            assert m8 == oracle.mbs_static_m8(float(a))
        # with that factor the FLOOR scale puts the macro maximum within one part in 256 below V
        if 0x0080 <= hbits:
            F = 1 + Fraction(m8, 256)
            s = oracle.elem_scale_exponent(fmt, float(a * F), "floor")
            y = a * F * Fraction(2) ** s
            assert V * Fraction(256, 257) < y <= V, (fmt, hbits, y)


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("rule", ["ocp", "floor", "oas"])
def test_elem_quantize_against_exact_rationals(oracle, fmt, rule):
    eb, mb, _, V, _ = SPEC[fmt]
    vals = grid(fmt)
    h = half_step_top(fmt)
    top = max(Fraction(2) ** e for e in range(-20, 20) if Fraction(2) ** e <= V)
    rng = np.random.default_rng(FORMATS.index(fmt) * 3 + ["ocp", "floor", "oas"].index(rule))
    x = synth.to_bf16_bits(rng.standard_t(3, (6, 256)) * np.exp2(rng.integers(-12, 12, (6, 1))))
    x[0, 5] = 0x8000  # -0
    x[1, 32:64] = 0   # an all-zero block
    for use_mbs in (False, True):
        codes, scales, words = oracle.elem_quantize(fmt, x, rule, mbs=use_mbs)
        for r in range(x.shape[0]):
            for g in range(2):
                xs = [bf16_frac(int(v)) for v in x[r, 128 * g:128 * g + 128]]
                F = Fraction(1)
                if use_mbs:
                    q = V / max(abs(v) for v in xs)
                    while q >= 2:
                        q /= 2
                    while q < 1:
                        q *= 2
                    m8 = int((q - 1) * 256)
                    assert words[r, g] == m8
                    F = 1 + Fraction(m8, 256)
                for b in range(4):
                    blk = xs[32 * b:32 * b + 32]
                    amax = max(abs(v) for v in blk) * F
                    E = int(scales[r, 4 * g + b])
                    if amax == 0:
                        assert E == 127
                    else:
                        y = amax * Fraction(2) ** (127 - E)  # scaled maximum under the stored scale
                        if rule == "floor":
                            assert V / 2 < y <= V
                        elif rule == "oas":
                            assert (V + h) / 2 < y <= V + h
                        else:
                            assert top <= y < 2 * top
                    for k, v in enumerate(blk):
                        c = int(codes[r, 128 * g + 32 * b + k])
                        want = nearest_code(vals, abs(v) * F * Fraction(2) ** (127 - E))
                        neg = bool(x[r, 128 * g + 32 * b + k] & 0x8000)
                        assert c == want | ((1 << (eb + mb)) if neg else 0), (fmt, rule, r, g, b, k)


def test_elem_e2m1_reproduces_the_mxfp4_quantizer(oracle):
    x = synth.activations_student_t(16, 512, 3.0, 0.01, 20.0, seed=5)
    for rule in ("ocp", "floor", "oas"):
        for use_mbs in (False, True):
            c4, s4, w4 = oracle.quantize(x, rule, mbs=use_mbs)
            c, s, w = oracle.elem_quantize("e2m1", x, rule, mbs=use_mbs)
            unpacked = np.empty(c.shape, np.uint8)
            unpacked[:, 0::2] = c4 & 15
            unpacked[:, 1::2] = c4 >> 4
            assert np.array_equal(c, unpacked) and np.array_equal(s, s4)
            assert (w is None and w4 is None) or np.array_equal(w, w4)
            assert np.array_equal(oracle.elem_dequantize("e2m1", c, s, w), oracle.dequantize(c4, s4, w4))
    a = oracle.quantize(x[:8], "oas", mbs=True)
    b = oracle.quantize(x[8:], "oas", mbs=True)
    ae = oracle.elem_quantize("e2m1", x[:8], "oas", mbs=True)
    be = oracle.elem_quantize("e2m1", x[8:], "oas", mbs=True)
    assert np.array_equal(oracle.elem_gemm("e2m1", ae, "e2m1", be), oracle.gemm(a, b))


def test_elem_special_values(oracle):
    x = np.zeros((1, 128), np.uint16)
    x[0, 3] = 0x7F80   # +Inf in block 0
    x[0, 40] = 0x7FC0  # NaN in block 1
    x[0, 70] = 0x3F80  # 1.0 in block 2
    for fmt in FORMATS:
        c, s, w = oracle.elem_quantize(fmt, x, "oas", mbs=True)
        assert s[0, 0] == 255 and s[0, 1] == 255 and not c[0, :64].any()
        # the macro maximum is taken over the finite elements: 1.0 -> V exactly
        V = SPEC[fmt][3]
        got = Fraction(oracle.elem_decode(fmt, int(c[0, 70]))) * Fraction(2) ** (int(s[0, 2]) - 127) / (1 + Fraction(int(w[0, 0]), 256))
        assert abs(got - 1) <= Fraction(1, 256)
        assert s[0, 3] == 127


# ------------------------------------------------------------------------------------------------
# dequantizer, GEMM, and the direction of the gains
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("fmt", FORMATS)
def test_elem_dequantize_and_gemm_against_numpy(oracle, fmt):
    rng = np.random.default_rng(3)
    xa = synth.to_bf16_bits(rng.standard_normal((5, 256)))
    xb = synth.to_bf16_bits(rng.standard_normal((7, 256)) * 0.05)
    a = oracle.elem_quantize(fmt, xa, "oas", mbs=True)
    b = oracle.elem_quantize("e4m3", xb, "floor", mbs=True)
    vals_a = np.array([oracle.elem_decode(fmt, c) for c in range(256)])
    vals_b = np.array([oracle.elem_decode("e4m3", c) for c in range(256)])

    def dq(t, vals):
        c, s, w = t
        return vals[c] * np.exp2(np.repeat(s.astype(np.float64), 32, 1) - 127) / (1 + np.repeat(w.astype(np.float64), 128, 1) / 256)

    da, db = dq(a, vals_a), dq(b, vals_b)
    assert np.allclose(oracle.elem_dequantize(fmt, *a), da, rtol=1e-15, atol=0)
    # one macro block at a time, as Sec. 4.3.2 applies the correction; fp64 throughout
    want = da @ db.T
    got = oracle.elem_gemm(fmt, a, "e4m3", b)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12 * np.abs(want).max())
    assert np.allclose(oracle.elem_gemm(fmt, a, "e4m3", b, rows=[4, 0]), want[[4, 0]], rtol=1e-12,
                       atol=1e-12 * np.abs(want).max())


def test_elem_qsnr_directions(oracle):
    """More element bits give a higher QSNR, and within every format MBS with OAS is at least as good as the
    OCP rule alone (directions only; no value of the paper covers these formats)."""
    x = synth.activations_student_t(64, 1024, 3.0, 0.01, 20.0, seed=11)
    ref = oracle.bf16_to_f64(x)

    def q(fmt, rule, mbs):
        return oracle.qsnr_db(ref, oracle.elem_dequantize(fmt, *oracle.elem_quantize(fmt, x, rule, mbs=mbs)))

    base = {f: q(f, "ocp", False) for f in ["e2m1", "e2m3", "e3m2", "e4m3", "e5m2"]}
    best = {f: q(f, "oas", True) for f in base}
    assert base["e2m1"] < base["e3m2"] < base["e2m3"]
    assert base["e5m2"] < base["e4m3"] and base["e2m1"] < base["e5m2"]
    for f in base:
        assert best[f] > base[f], (f, base[f], best[f])


# ------------------------------------------------------------------------------------------------
# MBS-Dynamic on the element formats (Sec. 4.3.3 with the true error; the candidate list is a parameter)
# ------------------------------------------------------------------------------------------------
def exact_sse(fmt, xs, m8, rule):
    """Sum of squared errors of one macro block (a list of bf16 patterns) under word m8, in exact rationals, with the
    block scale and the rounding worked out here from the specification's grid."""
    _, mb, _, V, _ = SPEC[fmt]
    vals = grid(fmt)
    h = half_step_top(fmt)
    top = max(Fraction(2) ** e for e in range(-20, 20) if Fraction(2) ** e <= V)
    F = 1 + Fraction(m8, 256)
    total = Fraction(0)
    for b in range(0, len(xs), 32):
        blk = [bf16_frac(int(v)) for v in xs[b:b + 32]]
        amax = max(abs(v) for v in blk) * F
        s = 0
        if amax > 0:
            # the power of two that takes amax into the rule's interval
            lo, hi, closed_low = {"floor": (V / 2, V, False), "oas": ((V + h) / 2, V + h, False), "ocp": (top, 2 * top, True)}[rule]
            while amax * Fraction(2) ** s > hi or (closed_low and amax * Fraction(2) ** s >= hi):
                s -= 1
            while amax * Fraction(2) ** s < lo or (not closed_low and amax * Fraction(2) ** s <= lo):
                s += 1
        for v in blk:
            q = vals[nearest_code(vals, abs(v) * F * Fraction(2) ** s)]
            x_hat = (q if v >= 0 else -q) / (F * Fraction(2) ** s)
            total += (x_hat - v) ** 2
    return total


@pytest.mark.parametrize("fmt", FORMATS)
def test_elem_mbs_sse_against_exact_rationals(oracle, fmt):
    rng = np.random.default_rng(60 + FORMATS.index(fmt))
    x = synth.to_bf16_bits(rng.standard_t(3, (3, 192)) * np.exp2(rng.integers(-10, 10, (3, 1))))  # a half macro block too
    for rule in ("ocp", "floor", "oas"):
        words = rng.integers(0, 256, (3, 2), dtype=np.uint8)
        got = oracle.elem_mbs_sse_rows(fmt, x, words, rule)
        for r in range(3):
            for g in range(2):
                want = exact_sse(fmt, x[r, 128 * g:128 * g + 128], int(words[r, g]), rule)
                assert abs(Fraction(got[r, g]) - want) <= want * Fraction(1, 10 ** 12), (fmt, rule, r, g)
    # and it is the error of what the quantizer and the dequantizer give for those words
    words = rng.integers(0, 256, (3, 2), dtype=np.uint8)
    c, s, _ = oracle.elem_quantize_given_mbs(fmt, x, words, "oas")
    err = oracle.elem_dequantize(fmt, c, s, words) - oracle.bf16_to_f64(x)
    sse = np.stack([(err[:, :128] ** 2).sum(1), (err[:, 128:] ** 2).sum(1)], 1)
    assert np.allclose(oracle.elem_mbs_sse_rows(fmt, x, words, "oas"), sse, rtol=1e-12, atol=0)


@pytest.mark.parametrize("fmt", FORMATS)
def test_elem_mbs_dynamic_is_the_brute_force_argmin(oracle, fmt):
    rng = np.random.default_rng(70 + FORMATS.index(fmt))
    x = synth.to_bf16_bits(rng.standard_t(3, (8, 384)) * 0.05)
    for rule, cands in (("oas", (0, 16, 16)), ("floor", (-3, 7, 5)), ("ocp", (0, 256, 1))):
        c, s, w = oracle.elem_quantize_mbs_dynamic(fmt, x, rule, *cands)
        static = oracle.elem_quantize(fmt, x, rule, mbs=True)[2]
        steps = [0] + [(cands[0] + j) * cands[2] for j in range(cands[1])]
        cand = np.stack([((static.astype(np.int64) + st) % 256).astype(np.uint8) for st in steps])
        sse = np.stack([oracle.elem_mbs_sse_rows(fmt, x, cw, rule) for cw in cand])
        first_min = sse.argmin(0)  # the first of equal minima: the static word, then the lowest j
        assert np.array_equal(w, np.take_along_axis(cand, first_min[None], 0)[0])
        oc, os_, _ = oracle.elem_quantize_given_mbs(fmt, x, w, rule)
        assert np.array_equal(c, oc) and np.array_equal(s, os_)
        assert (oracle.elem_mbs_sse_rows(fmt, x, w, rule) <= oracle.elem_mbs_sse_rows(fmt, x, static, rule)).all()
    # no candidates: MBS-Static
    c0, s0, w0 = oracle.elem_quantize_mbs_dynamic(fmt, x, "oas", 0, 0, 16)
    cs, ss, ws = oracle.elem_quantize(fmt, x, "oas", mbs=True)
    assert np.array_equal(c0, cs) and np.array_equal(s0, ss) and np.array_equal(w0, ws)
    # a window with a non-finite element keeps the static word; E2M1 through this route is the MXFP4 function
    y = x.copy()
    y[0, 7] = 0x7F80
    assert oracle.elem_quantize_mbs_dynamic(fmt, y, "oas")[2][0, 0] == oracle.elem_quantize(fmt, y, "oas", mbs=True)[2][0, 0]


def test_elem_mbs_dynamic_e2m1_reproduces_the_mxfp4_search(oracle):
    x = synth.gaussian(16, 512, 0.02, 9)
    c4, s4, w4 = oracle.quantize_mbs_dynamic(x, "oas")
    c, s, w = oracle.elem_quantize_mbs_dynamic("e2m1", x, "oas")
    assert np.array_equal(w, w4) and np.array_equal(s, s4)
    assert np.array_equal(c[:, 0::2] | (c[:, 1::2] << 4), c4)
    assert np.array_equal(oracle.elem_mbs_sse_rows("e2m1", x, w, "oas"), oracle.mbs_sse_rows(x, w, "oas"))


def test_elem_mbs_dynamic_qsnr_direction(oracle):
    """The searched word lowers the error of Gaussian weights in every format (Sec. 4.3.3: direction only; the size of
    the gain on these formats is this build's observation)."""
    x = synth.gaussian(64, 1024, 0.02, 11)
    ref = oracle.bf16_to_f64(x)
    for fmt in FORMATS:
        cs, ss, ws = oracle.elem_quantize(fmt, x, "oas", mbs=True)
        cd, sd, wd = oracle.elem_quantize_mbs_dynamic(fmt, x, "oas")
        qs = oracle.qsnr_db(ref, oracle.elem_dequantize(fmt, cs, ss, ws))
        qd = oracle.qsnr_db(ref, oracle.elem_dequantize(fmt, cd, sd, wd))
        assert qd > qs, (fmt, qs, qd)
