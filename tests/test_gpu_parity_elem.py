"""GPU parity for the 8-bit MX element formats (E4M3, E5M2): the HIP path through the C ABI against the CPU
oracle on the same seeded inputs.  Bar as for MXFP4: bit-exact codes, E8M0 scales and MBS words; GEMM on
quantized tensors within max|C - C_oracle| <= 1e-3 * RMS(C_oracle) on the fp32 output, and the bf16 output equal
to the rounding of the kernel's own fp32 output.  Uniformly random codes are held to a per-output bound derived
from how the matrix instruction adds FP8 products (see ABS_TOL), and sums that need no alignment must be exact.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

RULES = ("ocp", "floor", "oas")
ELEMS = ("e4m3", "e5m2")          # the 8-bit formats (one code per byte)
QUANT_ELEMS = ELEMS + ("e2m3", "e3m2")  # all four (6-bit codes packed)
MAX_CODE = {"e4m3": 0x7E, "e5m2": 0x7B}


def canonical_codes(elem, codes: np.ndarray) -> np.ndarray:
    """The oracle keeps one code per byte; the library packs 6-bit codes, element k of a row in bits 6k .. 6k+5."""
    if elem in ELEMS:
        return codes
    c = codes.reshape(codes.shape[0], -1, 4).astype(np.uint32)
    w = c[..., 0] | (c[..., 1] << 6) | (c[..., 2] << 12) | (c[..., 3] << 18)
    out = np.stack([w & 0xFF, (w >> 8) & 0xFF, (w >> 16) & 0xFF], axis=-1).astype(np.uint8)
    return out.reshape(codes.shape[0], -1)
GEMM_TOL = 1e-3


@pytest.fixture(scope="module")
def mx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2603_08713_amd as mx_

    mx_.load_library()
    return mx_


def dev_bf16(bits: np.ndarray):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def dev_u8(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return None if t is None else t.cpu().numpy()


def assert_quant_equal(mx, oracle, elem, bits, rule, mbs, what="", x=None):
    x = dev_bf16(bits) if x is None else x
    c, s, w = mx.mx_quantize_elem(x, elem, rule, use_mbs=mbs)
    torch.cuda.synchronize()
    oc, os_, ow = oracle.elem_quantize(elem, bits, rule, mbs=mbs)
    oc = canonical_codes(elem, oc)
    tag = "%s %s rule=%s mbs=%s" % (what, elem, rule, mbs)
    if mbs:
        bad = np.argwhere(host(w) != ow)
        assert bad.size == 0, "%s: %d MBS words differ, first at %s" % (tag, len(bad), bad[:3])
    bad = np.argwhere(host(s) != os_)
    assert bad.size == 0, "%s: %d scales differ, first at %s gpu=%s oracle=%s" % (
        tag, len(bad), bad[:3], host(s)[tuple(bad[0])], os_[tuple(bad[0])])
    bad = np.argwhere(host(c) != oc)
    assert bad.size == 0, "%s: %d codes differ, first at %s gpu=%#x oracle=%#x" % (
        tag, len(bad), bad[:3], host(c)[tuple(bad[0])], oc[tuple(bad[0])])


# ------------------------------------------------------------------------------------------------
# quantizer
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("hw", [1, 0])
@pytest.mark.parametrize("elem", QUANT_ELEMS)
def test_quantize_elem_tiny_config(mx, oracle, elem, hw):
    from paper_2603_08713_amd import synth

    with mx.forced(quantize_elem_hw=hw):
        a, w = synth.tiny(0)
        for rule in RULES:
            for mbs in (False, True):
                assert_quant_equal(mx, oracle, elem, a, rule, mbs, "tiny A")
                assert_quant_equal(mx, oracle, elem, w, rule, mbs, "tiny W")


@pytest.mark.parametrize("hw", [1, 0])
@pytest.mark.parametrize("elem", QUANT_ELEMS)
def test_quantize_elem_every_bf16_pattern(mx, oracle, elem, hw):
    """All 65536 bf16 patterns (subnormals, Inf, NaN, both zeros): in natural order (blocks of similar
    magnitude) and shuffled so that blocks mix magnitudes and elements land in every binade of the element
    format, its subnormals included; plus exact ties of every spacing."""
    with mx.forced(quantize_elem_hw=hw):
        allbits = np.arange(65536, dtype=np.uint16).reshape(128, 512)
        rng = np.random.default_rng(0)
        flat = allbits.reshape(-1)
        finite = flat[(flat & 0x7F80) != 0x7F80]
        mid = finite[((finite >> 7) & 0xFF > 100) & ((finite >> 7) & 0xFF < 150)]
        cases = {
            "natural": allbits,
            "shuffled-all": rng.permutation(flat).reshape(128, 512),
            "shuffled-mid": rng.choice(mid, size=(96, 1024)),
            "shuffled-finite": rng.choice(finite, size=(64, 640)),
        }
        # ties: odd multiples of half a spacing in every binade below a block maximum that is a power of two
        # (scale 2^-e under OCP), for binades from the top of the format down into its subnormals
        k = np.arange(1, 64, 2, dtype=np.float32)  # 32 odd numerators
        rows = []
        for e in range(0, 20):
            row = k * np.float32(2.0) ** (-e - 5)
            row[0] = 1.0  # the block maximum
            rows.append(row)
        t = np.stack(rows).astype(np.float32)
        tb = (t.view(np.uint32) >> 16).astype(np.uint16)
        assert np.array_equal((tb.astype(np.uint32) << 16).view(np.float32), t)
        tb[:, 1::2] |= 0x8000
        cases["ties"] = np.tile(tb, (1, 4))
        for name, bits in cases.items():
            for rule in RULES:
                for mbs in (False, True):
                    assert_quant_equal(mx, oracle, elem, bits, rule, mbs, name)


@pytest.mark.parametrize("rows,K,ld", [(1, 32, 32), (3, 96, 104), (5, 2880, 2880), (2, 4096 + 64, 4232), (7, 512, 512),
                                        (130, 160, 160)])
def test_quantize_elem_ragged_shapes(mx, oracle, rows, K, ld):
    from paper_2603_08713_amd import synth

    rng = np.random.default_rng(rows * 1000 + K)
    full = synth.to_bf16_bits(rng.standard_t(3, (rows, ld)))
    x = dev_bf16(full)[:, :K]
    for elem in QUANT_ELEMS:
        for rule, mbs in (("oas", True), ("ocp", False), ("floor", True)):
            assert_quant_equal(mx, oracle, elem, full[:, :K], rule, mbs, "ragged", x=x)


def test_quantize_elem_empty(mx):
    x = torch.empty((0, 128), dtype=torch.bfloat16, device="cuda")
    c, s, w = mx.mx_quantize_elem(x, "e4m3")
    assert c.shape == (0, 128) and s.shape == (0, 4) and w.shape == (0, 1)
    assert mx.mx_quantize_elem(x, "e2m3")[0].shape == (0, 96)


def test_quantize_elem_full_size_activation(mx, oracle):
    """Llama-3-8B FFN activation shape (4096 x 4096); every 8th row is checked against the oracle."""
    from paper_2603_08713_amd import synth

    a = synth.activations_student_t(4096, 4096, 4.0, 0.01, 20.0, 1)
    x = dev_bf16(a)
    for elem, rule in (("e4m3", "oas"), ("e5m2", "oas"), ("e4m3", "ocp"), ("e2m3", "oas"), ("e3m2", "oas")):
        c, s, w = mx.mx_quantize_elem(x, elem, rule, use_mbs=True)
        torch.cuda.synchronize()
        oc, os_, ow = oracle.elem_quantize(elem, a[::8], rule, mbs=True)
        assert np.array_equal(host(w)[::8], ow) and np.array_equal(host(s)[::8], os_)
        assert np.array_equal(host(c)[::8], canonical_codes(elem, oc))


# ------------------------------------------------------------------------------------------------
# dequantizer
# ------------------------------------------------------------------------------------------------
def to_bf16_bits_rne(f32: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(f32, np.float32).view(np.uint32)
    nan = np.isnan(f32)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    r[nan] = ((u[nan] >> 16) | 0x40).astype(np.uint16)
    return r


@pytest.mark.parametrize("elem", QUANT_ELEMS)
def test_dequantize_elem_matches_oracle(mx, oracle, elem):
    """Quantized heavy-tailed tensors, and every code under every scale byte and MBS word: the fp32 output equals
    the oracle's fp64 value rounded to fp32, the bf16 output that fp32 value rounded to nearest even; NaN blocks."""
    from paper_2603_08713_amd import synth

    x = synth.activations_student_t(37, 2880, 3.0, 0.01, 30.0, 21)
    x[3, 40] = 0x7F80  # a non-finite block
    cases = [oracle.elem_quantize(elem, x, "oas", mbs=True), oracle.elem_quantize(elem, x, "ocp", mbs=False)]
    rng = np.random.default_rng(5)
    rows, K = 256, 1024
    if elem in ELEMS:
        c = rng.integers(0, 256, (rows, K), dtype=np.uint8)
        mag = c & 0x7F
        c = np.where(mag > MAX_CODE[elem], (c & 0x80) | (mag & 0x3F), c).astype(np.uint8)
    else:
        c = rng.integers(0, 64, (rows, K), dtype=np.uint8)                    # every 6-bit code is a number
    s = np.repeat(np.arange(256, dtype=np.uint8)[:, None], K // 32, 1)       # row r: scale byte r (255: NaN)
    w = rng.integers(0, 256, (rows, K // 128), dtype=np.uint8)
    w[:, 0] = 0
    cases.append((c, s, w))
    for codes, scales, words in cases:
        with np.errstate(over="ignore"):  # the largest scale bytes overflow fp32 on both sides
            want = oracle.elem_dequantize(elem, codes, scales, words).astype(np.float32)
        dc, ds, dw = dev_u8(canonical_codes(elem, codes)), dev_u8(scales), dev_u8(words)
        got32 = host(mx.mx_dequantize_elem(elem, dc, ds, dw, "f32"))
        got16 = host(mx.mx_dequantize_elem(elem, dc, ds, dw, "bf16").view(torch.int16)).view(np.uint16)
        nan = np.isnan(want)
        assert np.array_equal(np.isnan(got32), nan)
        assert np.array_equal(got32.view(np.uint32)[~nan], want.view(np.uint32)[~nan])
        assert np.array_equal(got16[~nan], to_bf16_bits_rne(want)[~nan])
        assert np.all((got16[nan] & 0x7F80) == 0x7F80) and np.all((got16[nan] & 0x7F) != 0)
    # strided output and an odd column offset (element stores)
    codes, scales, words = cases[0]
    big = torch.zeros((37, 2880 + 9), dtype=torch.float32, device="cuda")
    packed = dev_u8(canonical_codes(elem, codes))
    mx.mx_dequantize_elem(elem, packed, dev_u8(scales), dev_u8(words), "f32", out=big[:, 1:2881])
    ref = mx.mx_dequantize_elem(elem, packed, dev_u8(scales), dev_u8(words), "f32")
    ok = ~torch.isnan(ref)
    assert torch.equal(big[:, 1:2881][ok], ref[ok]) and float(big[:, 0].abs().max()) == 0.0 and float(big[:, 2881:].abs().max()) == 0.0


# ------------------------------------------------------------------------------------------------
# MBS-Dynamic
# ------------------------------------------------------------------------------------------------
def assert_elem_dynamic_valid(mx, oracle, elem, bits, rule="oas", what="", cands=(0, 16, 16)):
    """The kernel sums squared errors in fp32, the oracle (Sec. 4.3.3, Eq. 6 with the true error) in fp64, so near-ties
    may fall either way: what is unique is compared, the rest is checked for validity.
      * the chosen word is the static word or one of the candidates;
      * its exact sum of squared errors is within 1e-5 of the least one on offer, and where the least one is
        separated from the runner-up by more than 1e-4 the word itself is the oracle's;
      * windows the entry point documents as not searched (Inf/NaN inside, absmax outside [2^-63, 2^123)) keep the
        static word;
      * codes and scales are, bit for bit, those of the chosen word."""
    c, s, w = mx.mx_quantize_elem_mbs_dynamic(dev_bf16(bits), elem, rule, *cands)
    torch.cuda.synchronize()
    gw, gs, gc = host(w), host(s), host(c)
    tag = "%s %s rule=%s cands=%s" % (what, elem, rule, cands)
    static = oracle.elem_quantize(elem, bits, rule, mbs=True)[2]
    steps = [0] + [(cands[0] + j) * cands[2] for j in range(cands[1])]
    cand = np.stack([((static.astype(np.int64) + st) % 256).astype(np.uint8) for st in steps])
    sse = np.stack([oracle.elem_mbs_sse_rows(elem, bits, cw, rule) for cw in cand])
    rows, K = bits.shape
    nmac = static.shape[1]
    pad = np.zeros((rows, nmac * 128), np.float64)
    val = oracle.bf16_to_f64(bits)
    pad[:, :K] = np.where(np.isfinite(val), np.abs(val), 0.0)
    absmax = pad.reshape(rows, nmac, 128).max(2)
    searched = (sse[0] >= 0) & (absmax >= 2.0 ** -63) & (absmax < 2.0 ** 123)
    assert (cand == gw[None]).any(0).all(), "%s: a chosen word is not a candidate" % tag
    bad = np.argwhere(~searched & (gw != static))
    assert bad.size == 0, "%s: %d windows outside the searched domain left the static word, first %s" % (tag, len(bad), bad[:3])
    got = oracle.elem_mbs_sse_rows(elem, bits, gw, rule)
    best = sse.min(0)
    bad = np.argwhere(searched & (got > best * (1 + 1e-5)))
    assert bad.size == 0, "%s: %d windows miss the least SSE, first %s got %s best %s" % (
        tag, len(bad), bad[:3], got[tuple(bad[0])], best[tuple(bad[0])])
    ow = oracle.elem_quantize_mbs_dynamic(elem, bits, rule, *cands)[2]
    others = np.where(cand == ow[None], np.inf, sse)
    clear = searched & (others.min(0) > best * (1 + 1e-4))
    bad = np.argwhere(clear & (gw != ow))
    assert bad.size == 0, "%s: %d clearly separated windows differ from the oracle's word, first %s" % (tag, len(bad), bad[:3])
    oc, os_, _ = oracle.elem_quantize_given_mbs(elem, bits, gw, rule)
    for name, g, want in (("scales", gs, os_), ("code bytes", gc, canonical_codes(elem, oc))):
        bad = np.argwhere(g != want)
        assert bad.size == 0, "%s: %d %s differ from those of the chosen word, first at %s gpu=%s oracle=%s" % (
            tag, len(bad), name, bad[:3], g[tuple(bad[0])], want[tuple(bad[0])])
    return gw, float(clear.mean())


@pytest.mark.parametrize("elem", QUANT_ELEMS)
def test_quantize_elem_dynamic(mx, oracle, elem):
    """MBS-Dynamic on every element format and rule: Gaussian weights and heavy-tailed rows (several chunks of 512
    per row and a ragged tail with a half macro block), a list of candidates that passes the static word again,
    none at all, and all 255 other words."""
    from paper_2603_08713_amd import synth

    w_bits = synth.gaussian(24, 1216, 0.02, 21)
    t_bits = synth.activations_student_t(9, 2880, 3.0, 0.01, 20.0, 22)
    moved = 0.0
    for rule in RULES:
        gw, clear = assert_elem_dynamic_valid(mx, oracle, elem, w_bits, rule, "weights")
        static = oracle.elem_quantize(elem, w_bits, rule, mbs=True)[2]
        moved = max(moved, float((gw != static).mean()))
        assert clear > 0.5  # most windows have a clear winner: the comparison of words is not vacuous
        assert_elem_dynamic_valid(mx, oracle, elem, t_bits, rule, "student-t", (-3, 9, 7))
    assert moved > 0.3      # and the search does move words
    assert_elem_dynamic_valid(mx, oracle, elem, w_bits[:4], "oas", "all words", (1, 255, 1))
    # no candidates: MBS-Static, bit for bit
    c, s, w = mx.mx_quantize_elem_mbs_dynamic(dev_bf16(w_bits), elem, "oas", 0, 0, 16)
    c0, s0, w0 = mx.mx_quantize_elem(dev_bf16(w_bits), elem, "oas")
    assert torch.equal(c, c0) and torch.equal(s, s0) and torch.equal(w, w0)
    # the searched words lower the weights' error, and the GEMM consumes them unchanged
    wk = np.ascontiguousarray(w_bits[:, :1152])
    qs, qd = mx.mx_quantize_elem(dev_bf16(wk), elem, "oas"), mx.mx_quantize_elem_mbs_dynamic(dev_bf16(wk), elem, "oas")
    ref = oracle.bf16_to_f64(wk)
    q_static = oracle.qsnr_db(ref, host(mx.mx_dequantize_elem(elem, *qs, "f32")).astype(np.float64))
    q_dynamic = oracle.qsnr_db(ref, host(mx.mx_dequantize_elem(elem, *qd, "f32")).astype(np.float64))
    assert q_dynamic > q_static, (elem, q_static, q_dynamic)
    a_bits = synth.activations_student_t(64, 1152, 3.0, 0.01, 20.0, 23)
    qa = mx.mx_quantize_elem(dev_bf16(a_bits), elem, "oas")
    oa = oracle.elem_quantize(elem, a_bits, "oas", mbs=True)
    ob = oracle.elem_quantize_given_mbs(elem, wk, host(qd[2]), "oas")
    assert_gemm_close(host(mx.mx_gemm_mbs_elem(elem, *qa, elem, *qd, "f32")), oracle.elem_gemm(elem, oa, elem, ob), "dynamic words %s" % elem)


@pytest.mark.parametrize("elem", QUANT_ELEMS)
def test_quantize_elem_dynamic_edge_cases(mx, oracle, elem):
    """Zero windows, Inf and NaN, subnormal and huge magnitudes, a zero block beside a large one, blocks more than
    30 binades apart, a strided input."""
    rng = np.random.default_rng(24)
    x = np.zeros((12, 512), np.uint16)
    x[0] = 0                                            # all zero
    x[1, ::7] = 0x0001                                  # smallest subnormals
    x[2] = rng.integers(0x0001, 0x0080, 512)            # subnormal magnitudes
    x[3] = rng.integers(0x7E00, 0x7F80, 512)            # the largest binades
    x[4] = rng.integers(0x3C00, 0x4000, 512); x[4, 5] = 0x7F80; x[4, 300] = 0xFFC0   # Inf, NaN
    x[5] = rng.integers(0x3C00, 0x4000, 512); x[5, 128:160] = 0                       # a zero block
    x[6] = rng.integers(0x3C00, 0x4000, 512); x[6, 32:64] = rng.integers(0x1000, 0x1080, 32)  # ~88 binades below
    x[7] = rng.integers(0x0000, 0x7F80, 512) | (rng.integers(0, 2, 512) << 15)        # anything finite, both signs
    x[8] = rng.integers(0x1F80, 0x2100, 512)            # around 2^-63, the lower end of the searched domain
    x[9] = rng.integers(0x7C80, 0x7E00, 512)            # around 2^123, the upper end
    x[10] = rng.integers(0x3F80, 0x4000, 512) | 0x8000  # all negative
    x[11] = 0x3F80                                      # all equal
    for rule in RULES:
        assert_elem_dynamic_valid(mx, oracle, elem, x, rule, "edge cases")
    # strided input and preallocated outputs
    big = torch.zeros((12, 640), dtype=torch.bfloat16, device="cuda")
    big[:, :512] = dev_bf16(x)
    c, s, w = mx.mx_quantize_elem_mbs_dynamic(big[:, :512], elem, "oas")
    c1, s1, w1 = mx.mx_quantize_elem_mbs_dynamic(dev_bf16(x), elem, "oas")
    assert torch.equal(c, c1) and torch.equal(s, s1) and torch.equal(w, w1)


# ------------------------------------------------------------------------------------------------
# GEMM
# ------------------------------------------------------------------------------------------------
def random_operand(rng, elem, rows, K, lo=110, hi=140):
    """Uniformly random finite codes, a spread of E8M0 bytes, random MBS words."""
    c = rng.integers(0, 256, (rows, K), dtype=np.uint8)
    mag = c & 0x7F
    c = np.where(mag > MAX_CODE[elem], (c & 0x80) | (mag & 0x3F), c).astype(np.uint8)
    return (c, rng.integers(lo, hi, (rows, K // 32), dtype=np.uint8), rng.integers(0, 256, (rows, (K + 127) // 128), dtype=np.uint8))


def gpu_gemm(mx, ea, a, eb, b, out_dtype="f32", out=None, kernel=2):
    """kernel: 2 = the main kernel in the form the problem allows (what most tests here are about), 1 = its general
    form, 3 = the few-row kernel, None = whatever the library picks."""
    da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
    if kernel is None:
        return mx.mx_gemm_mbs_elem(ea, da[0], da[1], da[2], eb, db[0], db[1], db[2], out_dtype, out=out)
    with mx.forced(gemm_elem=kernel):
        return mx.mx_gemm_mbs_elem(ea, da[0], da[1], da[2], eb, db[0], db[1], db[2], out_dtype, out=out)


def assert_gemm_close(got, want, what=""):
    rms = float(np.sqrt(np.mean(want ** 2)))
    err = float(np.max(np.abs(got.astype(np.float64) - want)))
    assert err <= GEMM_TOL * rms, "%s: max err %.3e vs %.3e (rms %.3e)" % (what, err, GEMM_TOL * rms, rms)


# The accumulation contract of mx_gemm_mbs_elem (include/mx4.h) has two bounds.  (1) Quantized tensors, and any
# operands whose products stay within 2^13 of each other inside a group of 16 K-elements: the 1e-3 * RMS bar of
# the MXFP4 GEMM (GEMM_TOL; the tests on quantized tensors and on E2M3 codes below).  (2) Any codes and scale
# bytes: |C - exact| <= 2^-11 * sum_k |a_ik| |b_jk| per output, the secondary bound, because the matrix
# instruction aligns the products of such a group to the group's largest exponent and cuts them off about 13
# bits below it.  ABS_TOL is bound (2); it is used only on uniformly random codes under scale bytes spread over
# 30 binades, which bound (1) does not cover (the largest ratio seen there is below 2^-13).
ABS_TOL = 2.0 ** -11


def assert_gemm_within_abs_bound(oracle, got, ea, a, eb, b, what=""):
    want = oracle.elem_gemm(ea, a, eb, b)
    absc = oracle.elem_gemm(ea, (a[0] & 0x7F, a[1], a[2]), eb, (b[0] & 0x7F, b[1], b[2]))
    ratio = np.abs(got.astype(np.float64) - want) / absc
    assert float(np.nanmax(ratio)) <= ABS_TOL, "%s: max |err| / sum|a||b| = %.3e" % (what, float(np.nanmax(ratio)))


@pytest.mark.parametrize("ea,eb", [("e4m3", "e4m3"), ("e4m3", "e5m2"), ("e5m2", "e4m3"), ("e5m2", "e5m2")])
def test_gemm_elem_random_codes_and_scales(mx, oracle, ea, eb):
    """Exercises every code, scale byte and lane position of the operand layout; shapes span several tiles of
    256 x 128 with ragged tails, K several turns of the three-slot ring plus each remainder."""
    rng = np.random.default_rng(42)
    hi = 132 if "e5m2" in (ea, eb) else 140  # keep |C| inside fp32 with E5M2's 2^15
    # (K % 512 == 0 takes the kernel's fast form: 1, 2, 3 and 4 groups of four stages, then one turn of the loop,
    # and one turn plus one and plus two groups)
    for (M, N, K) in ((16, 16, 128), (64, 48, 256), (130, 200, 384), (257, 129, 1024), (300, 260, 640), (520, 390, 896),
                      (40, 200, 512), (257, 130, 1536), (100, 129, 2048), (70, 140, 6144), (33, 260, 6656), (260, 33, 7168),
                      # K ending with half a macro block (general form; rows of E8M0 bytes on even addresses only)
                      (130, 200, 192), (257, 129, 1216), (300, 140, 2880)):
        a, b = random_operand(rng, ea, M, K, 110, hi), random_operand(rng, eb, N, K, 110, hi)
        assert_gemm_within_abs_bound(oracle, host(gpu_gemm(mx, ea, a, eb, b)), ea, a, eb, b, "mbs %dx%dx%d" % (M, N, K))
        for a1, b1, name in (((a[0], a[1], None), b, "B words only"), (a, (b[0], b[1], None), "A words only"),
                             ((a[0], a[1], None), (b[0], b[1], None), "no words")):
            assert_gemm_within_abs_bound(oracle, host(gpu_gemm(mx, ea, a1, eb, b1)), ea, a1, eb, b1,
                                         "%s %dx%dx%d" % (name, M, N, K))


@pytest.mark.parametrize("ea,eb", [("e2m3", "e2m3"), ("e2m3", "e3m2"), ("e3m2", "e2m3"), ("e3m2", "e3m2")])
def test_gemm_elem_six_bit_random_codes_and_scales(mx, oracle, ea, eb):
    """MXFP6 operands (packed 6-bit codes; every code is a finite value): every code, scale byte and lane position;
    tiles with ragged tails; K of 1 to 4 groups of four stages, one turn of the loop, and a turn plus one and two
    groups; K % 512 != 0 takes the general form (1, 3, 5, 7 and 13 stages).  E2M3 products span 12 binades and add up without loss, like FP4's; with E3M2 (18 binades) the bound
    of the 8-bit formats applies."""
    rng = np.random.default_rng(46)
    for (M, N, K) in ((16, 16, 512), (257, 130, 1536), (100, 129, 2048), (300, 260, 1024), (70, 140, 6144), (33, 260, 6656),
                      (260, 33, 7168), (16, 16, 128), (130, 200, 384), (300, 260, 640), (520, 390, 896), (257, 129, 1664),
                      # K ending with half a macro block: the last stage holds 48 of its 96 bytes per row
                      (130, 200, 192), (257, 129, 1216), (300, 140, 2880)):
        a = (rng.integers(0, 64, (M, K), dtype=np.uint8), rng.integers(110, 140, (M, K // 32), dtype=np.uint8),
             rng.integers(0, 256, (M, (K + 127) // 128), dtype=np.uint8))
        b = (rng.integers(0, 64, (N, K), dtype=np.uint8), rng.integers(110, 140, (N, K // 32), dtype=np.uint8),
             rng.integers(0, 256, (N, (K + 127) // 128), dtype=np.uint8))
        for a1, b1, name in ((a, b, "mbs"), ((a[0], a[1], None), b, "B words only"), ((a[0], a[1], None), (b[0], b[1], None), "no words")):
            pa, pb = (canonical_codes(ea, a1[0]), a1[1], a1[2]), (canonical_codes(eb, b1[0]), b1[1], b1[2])
            got = host(gpu_gemm(mx, ea, pa, eb, pb))
            want = oracle.elem_gemm(ea, a1, eb, b1)
            if ea == "e2m3" and eb == "e2m3":
                assert_gemm_close(got, want, "%s %s x %s %dx%dx%d" % (name, ea, eb, M, N, K))
            else:
                absc = oracle.elem_gemm(ea, (a1[0] & 0x1F, a1[1], a1[2]), eb, (b1[0] & 0x1F, b1[1], b1[2]))
                ratio = float(np.nanmax(np.abs(got.astype(np.float64) - want) / absc))
                assert ratio <= ABS_TOL, "%s %s x %s %dx%dx%d: %.3e" % (name, ea, eb, M, N, K, ratio)
    with pytest.raises(mx.MxError) as e:  # 6-bit with 8-bit operands
        gpu_gemm(mx, "e2m3", (canonical_codes("e2m3", a[0]), a[1], a[2]), "e4m3", b)
    assert e.value.status == -4


def test_gemm_elem_six_bit_quantized_tensors(mx, oracle):
    """MXFP6 end to end on the GPU (quantize both operands, multiply) against the oracle: operands bit-exact, the
    product within 1e-3 RMS, a second launch bit-identical, and QSNR(AB) between MXFP4's and MXFP8's."""
    from paper_2603_08713_amd import synth

    M, N, K = 200, 300, 1536
    a_bits = synth.activations_student_t(M, K, 3.0, 0.01, 20.0, 3)
    w_bits = synth.gaussian(N, K, 0.02, 4)
    xa, xw = dev_bf16(a_bits), dev_bf16(w_bits)
    ref = oracle.matmul_bf16(a_bits, w_bits)
    q = {}
    for ea, eb, rule in (("e2m3", "e2m3", "oas"), ("e3m2", "e2m3", "floor"), ("e2m3", "e3m2", "ocp"), ("e3m2", "e3m2", "oas")):
        a = mx.mx_quantize_elem(xa, ea, rule)
        b = mx.mx_quantize_elem(xw, eb, rule)
        c = mx.mx_gemm_mbs_elem(ea, a[0], a[1], a[2], eb, b[0], b[1], b[2], "f32")
        c2 = mx.mx_gemm_mbs_elem(ea, a[0], a[1], a[2], eb, b[0], b[1], b[2], "f32")
        c16 = mx.mx_gemm_mbs_elem(ea, a[0], a[1], a[2], eb, b[0], b[1], b[2], "bf16")
        torch.cuda.synchronize()
        assert torch.equal(c, c2) and torch.equal(c16, c.to(torch.bfloat16))
        oa, ob = oracle.elem_quantize(ea, a_bits, rule, mbs=True), oracle.elem_quantize(eb, w_bits, rule, mbs=True)
        assert np.array_equal(host(a[0]), canonical_codes(ea, oa[0])) and np.array_equal(host(b[0]), canonical_codes(eb, ob[0]))
        assert_gemm_close(host(c), oracle.elem_gemm(ea, oa, eb, ob), "%s x %s %s" % (ea, eb, rule))
        q[(ea, eb, rule)] = oracle.qsnr_db(ref, host(c))
    a4, b4 = mx.mx_quantize_mbs(xa, "oas"), mx.mx_quantize_mbs(xw, "oas")
    q4 = oracle.qsnr_db(ref, host(mx.mx_gemm_mbs(*a4, *b4, "f32")))
    a8, b8 = mx.mx_quantize_elem(xa, "e4m3", "oas"), mx.mx_quantize_elem(xw, "e4m3", "oas")
    q8 = oracle.qsnr_db(ref, host(mx.mx_gemm_mbs_elem("e4m3", *a8, "e4m3", *b8, "f32")))
    assert q4 + 5.0 < q[("e2m3", "e2m3", "oas")] < q8 + 1.0, (q4, q, q8)


def test_gemm_elem_general_form_equals_fast_form(mx, oracle):
    """Where both forms of the kernel apply they run the same matrix instructions on the same data in the same
    order: bit-identical results."""
    rng = np.random.default_rng(45)
    for (M, N, K) in ((300, 200, 512), (257, 390, 2048), (64, 128, 6656)):
        a, b = random_operand(rng, "e4m3", M, K, 118, 136), random_operand(rng, "e5m2", N, K, 118, 132)
        a6 = (canonical_codes("e3m2", a[0] & 0x3F), a[1], a[2])
        b6 = (canonical_codes("e2m3", b[0] & 0x3F), b[1], b[2])
        for words in (True, False):
            for ea, a1, eb, b1 in (("e4m3", a, "e5m2", b), ("e3m2", a6, "e2m3", b6)):
                a1 = a1 if words else (a1[0], a1[1], None)
                b1 = b1 if words else (b1[0], b1[1], None)
                fast = gpu_gemm(mx, ea, a1, eb, b1)
                general = gpu_gemm(mx, ea, a1, eb, b1, kernel=1)
                assert torch.equal(fast, general), (ea, M, N, K, words)


def test_gemm_elem_general_form_at_full_size_repeats_bit_for_bit(mx):
    """The general form's stage waits count the loads a wavefront has issued; a count that does not match the
    loads made (without MBS words two fewer) lets a stage read codes that have not landed, now and then.  At the
    benchmark's shape, every tile in flight, repeated launches of either variant give the fast form's bits."""
    from paper_2603_08713_amd import synth

    M, N, K = 4096, 14336, 4096
    a_bits, w_bits = synth.llama8b_ffn_up(M, N, K)
    a = mx.mx_quantize_elem(dev_bf16(a_bits), "e4m3", "oas")
    b = mx.mx_quantize_elem(dev_bf16(w_bits), "e4m3", "oas")
    for words in (True, False):
        args = ("e4m3", a[0], a[1], a[2] if words else None, "e4m3", b[0], b[1], b[2] if words else None, "bf16")
        fast = mx.mx_gemm_mbs_elem(*args)
        with mx.forced(gemm_elem=1):
            for rep in range(5):
                assert torch.equal(mx.mx_gemm_mbs_elem(*args), fast), (words, rep)


ALL_PAIRS = [("e4m3", "e4m3"), ("e4m3", "e5m2"), ("e5m2", "e4m3"), ("e5m2", "e5m2"),
             ("e2m3", "e2m3"), ("e2m3", "e3m2"), ("e3m2", "e2m3"), ("e3m2", "e3m2")]


def random_operand_any(rng, elem, rows, K, lo=110, hi=140):
    """random_operand for any of the four formats: (codes one per byte for the oracle, codes as the library takes them)."""
    if elem in ELEMS:
        op = random_operand(rng, elem, rows, K, lo, hi)
        return op, op
    op = (rng.integers(0, 64, (rows, K), dtype=np.uint8), rng.integers(lo, hi, (rows, K // 32), dtype=np.uint8),
          rng.integers(0, 256, (rows, (K + 127) // 128), dtype=np.uint8))
    return op, (canonical_codes(elem, op[0]), op[1], op[2])


def assert_gemm_elem_ok(oracle, got, ea, a, eb, b, what, rows=None):
    """Bound (1) of the accumulation contract where it applies to random codes (E2M3 x E2M3), else bound (2)."""
    want = oracle.elem_gemm(ea, a, eb, b, rows=rows)
    if ea == "e2m3" and eb == "e2m3":
        return assert_gemm_close(got, want, what)
    keep = 0x7F if ea in ELEMS else 0x1F
    absc = oracle.elem_gemm(ea, (a[0] & keep, a[1], a[2]), eb, (b[0] & keep, b[1], b[2]), rows=rows)
    ratio = float(np.nanmax(np.abs(got.astype(np.float64) - want) / absc))
    assert ratio <= ABS_TOL, "%s: max |err| / sum|a||b| = %.3e" % (what, ratio)


@pytest.mark.parametrize("ea,eb", ALL_PAIRS)
def test_gemm_elem_few_rows(mx, oracle, ea, eb):
    """The few-row kernel (weights streamed once, K split over the wavefronts of a workgroup): every row count's
    fragment arrangement, ragged N, K of one group of four macro blocks up to the largest, every code, scale byte
    and lane position of the 16x16x128 instruction's operand layout; with and without MBS words on either side."""
    rng = np.random.default_rng(50)
    hi = 132 if "e5m2" in (ea, eb) else 140
    for (M, N, K) in ((1, 16, 512), (16, 100, 1024), (7, 8200, 512), (17, 130, 4096), (32, 48, 1536), (33, 70, 2560), (64, 40, 8192)):
        (a, pa), (b, pb) = random_operand_any(rng, ea, M, K, 110, hi), random_operand_any(rng, eb, N, K, 110, hi)
        for wa, wb in ((True, True), (False, True), (True, False), (False, False)):
            a1, b1 = (a[0], a[1], a[2] if wa else None), (b[0], b[1], b[2] if wb else None)
            pa1, pb1 = (pa[0], pa[1], pa[2] if wa else None), (pb[0], pb[1], pb[2] if wb else None)
            got = gpu_gemm(mx, ea, pa1, eb, pb1, kernel=3)
            assert_gemm_elem_ok(oracle, host(got), ea, a1, eb, b1, "few rows %s x %s %dx%dx%d words %d%d" % (ea, eb, M, N, K, wa, wb))
            if (wa, wb) == (True, True):
                # what the library picks for this shape is this kernel, and bf16 is the rounding of its fp32
                assert torch.equal(gpu_gemm(mx, ea, pa1, eb, pb1, kernel=None), got)
                assert torch.equal(gpu_gemm(mx, ea, pa1, eb, pb1, "bf16", kernel=None), got.to(torch.bfloat16))
    # a strided C with an odd column offset
    big = torch.zeros((M, N + 5), dtype=torch.float32, device="cuda")
    gpu_gemm(mx, ea, pa1, eb, pb1, out=big[:, 3:N + 3], kernel=3)
    assert torch.equal(big[:, 3:N + 3], got) and float(big[:, :3].abs().max()) == 0.0 and float(big[:, N + 3:].abs().max()) == 0.0
    # outside the kernel's range the request for it is refused, and the library takes the main kernel
    (a, pa), (b, pb) = random_operand_any(rng, ea, 65, 512, 120, 130), random_operand_any(rng, eb, 32, 512, 120, 130)
    with pytest.raises(mx.MxError) as e:
        gpu_gemm(mx, ea, pa, eb, pb, kernel=3)
    assert e.value.status == -1
    assert torch.equal(gpu_gemm(mx, ea, pa, eb, pb, kernel=None), gpu_gemm(mx, ea, pa, eb, pb, kernel=2))


def test_gemm_elem_few_rows_quantized_decode_shape(mx, oracle):
    """Decode shape (16 activation rows against a 4096 x 4096 weight), operands quantized on the GPU with OAS and
    MBS-Static in E4M3 and in E2M3: the whole output against the oracle at the 1e-3 RMS bar, and against the main
    kernel's."""
    from paper_2603_08713_amd import synth

    M, N, K = 16, 4096, 4096
    a_bits = synth.activations_student_t(M, K, 4.0, 0.01, 20.0, 3)
    w_bits = synth.gaussian(N, K, 0.02, 2)
    xa, xw = dev_bf16(a_bits), dev_bf16(w_bits)
    for elem in ("e4m3", "e2m3"):
        a, b = mx.mx_quantize_elem(xa, elem, "oas"), mx.mx_quantize_elem(xw, elem, "oas")
        c = mx.mx_gemm_mbs_elem(elem, *a, elem, *b, "f32")
        with mx.forced(gemm_elem=2):
            c_main = mx.mx_gemm_mbs_elem(elem, *a, elem, *b, "f32")
        oa, ob = oracle.elem_quantize(elem, a_bits, "oas", mbs=True), oracle.elem_quantize(elem, w_bits, "oas", mbs=True)
        want = oracle.elem_gemm(elem, oa, elem, ob)
        assert_gemm_close(host(c), want, "decode %s" % elem)
        assert_gemm_close(host(c_main), want, "decode %s, main kernel" % elem)


@pytest.mark.parametrize("ea,eb", [("e4m3", "e5m2"), ("e5m2", "e4m3"), ("e2m3", "e3m2"), ("e3m2", "e2m3")])
def test_gemm_elem_grouped(mx, oracle, ea, eb):
    """Grouped form: groups of 0, 1, a few, exactly one tile-row and several tile-rows of rows, each against its own
    weight; rows past the last group stay untouched; the same through mx_gemm_mbs_elem group by group."""
    rng = np.random.default_rng(51)
    hi = 132 if "e5m2" in (ea, eb) else 140
    N, K = 200, 640
    sizes = [0, 1, 37, 256, 0, 300, 5, 513]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    total, G = int(offs[-1]) + 9, len(sizes)
    (a, pa), (b, pb) = random_operand_any(rng, ea, total, K, 112, hi), random_operand_any(rng, eb, G * N, K, 112, hi)
    for wa, wb in ((True, True), (False, False), (True, False)):
        pa1, pb1 = (pa[0], pa[1], pa[2] if wa else None), (pb[0], pb[1], pb[2] if wb else None)
        da, db = [dev_u8(t) for t in pa1], [dev_u8(t) for t in pb1]
        out = torch.full((total, N), -7.0, dtype=torch.float32, device="cuda")
        mx.mx_gemm_mbs_elem_grouped(ea, da[0], da[1], da[2], eb, db[0], db[1], db[2], torch.from_numpy(offs).cuda(), N, "f32", out=out)
        got = host(out)
        assert np.all(got[offs[-1]:] == -7.0)
        for e in range(G):
            lo, hi_ = int(offs[e]), int(offs[e + 1])
            if lo == hi_:
                continue
            a_e = tuple(None if t is None else t[lo:hi_] for t in (a[0], a[1], a[2] if wa else None))
            b_e = tuple(None if t is None else t[e * N:(e + 1) * N] for t in (b[0], b[1], b[2] if wb else None))
            assert_gemm_elem_ok(oracle, got[lo:hi_], ea, a_e, eb, b_e, "group %d (%d rows) words %d%d" % (e, hi_ - lo, wa, wb))
            # the ungrouped entry point's general form runs the same instructions in the same order
            pa_e = tuple(None if t is None else t[lo:hi_] for t in pa1)
            pb_e = tuple(None if t is None else t[e * N:(e + 1) * N] for t in pb1)
            assert np.array_equal(host(gpu_gemm(mx, ea, pa_e, eb, pb_e, kernel=1)), got[lo:hi_]), e
    out16 = torch.zeros((total, N), dtype=torch.bfloat16, device="cuda")
    mx.mx_gemm_mbs_elem_grouped(ea, da[0], da[1], da[2], eb, db[0], db[1], db[2], torch.from_numpy(offs).cuda(), N, "bf16", out=out16)
    assert torch.equal(out16[:offs[-1]], out[:offs[-1]].to(torch.bfloat16))
    # no groups: nothing is written
    out.fill_(-7.0)
    mx.mx_gemm_mbs_elem_grouped(ea, da[0], da[1], da[2], eb, db[0][:0], db[1][:0], None, torch.zeros(1, dtype=torch.int64, device="cuda"), N, "f32", out=out)
    assert float((out + 7.0).abs().max()) == 0.0


def test_gemm_elem_grouped_many_groups(mx, oracle):
    """More groups than a wavefront has lanes, empty ones at the start, across the 64th and at the end: every group
    equals the ungrouped entry point's general form on its rows and weight, bit for bit, and the oracle on a few."""
    rng = np.random.default_rng(52)
    ea = eb = "e4m3"
    G, N, K = 70, 72, 256
    sizes = rng.integers(1, 30, G)
    sizes[[0, 1, 62, 63, 64, 65, 69]] = 0
    sizes[7], sizes[67] = 270, 129
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    total = int(offs[-1])
    (a, pa), (b, pb) = random_operand_any(rng, ea, total, K, 112, 140), random_operand_any(rng, eb, G * N, K, 112, 140)
    da, db = [dev_u8(t) for t in pa], [dev_u8(t) for t in pb]
    out = torch.full((total + 2, N), -7.0, dtype=torch.float32, device="cuda")
    mx.mx_gemm_mbs_elem_grouped(ea, da[0], da[1], da[2], eb, db[0], db[1], db[2], torch.from_numpy(offs).cuda(), N, "f32", out=out[:total])
    got = host(out)
    assert np.all(got[total:] == -7.0)
    for e in range(G):
        lo, hi_ = int(offs[e]), int(offs[e + 1])
        if lo == hi_:
            continue
        pa_e, pb_e = tuple(t[lo:hi_] for t in pa), tuple(t[e * N:(e + 1) * N] for t in pb)
        assert np.array_equal(host(gpu_gemm(mx, ea, pa_e, eb, pb_e, kernel=1)), got[lo:hi_]), e
        if e in (2, 7, 61, 66, 67, 68):
            assert_gemm_elem_ok(oracle, got[lo:hi_], ea, tuple(t[lo:hi_] for t in a), eb, tuple(t[e * N:(e + 1) * N] for t in b), "group %d" % e)


@pytest.mark.parametrize("ea,eb", [("e4m3", "e4m3"), ("e2m3", "e3m2")])
def test_gemm_elem_grouped_k_ending_in_half_a_macro_block(mx, oracle, ea, eb):
    """The MoE configuration's K = 2880 = 22.5 macro blocks, grouped: rows of E8M0 bytes are 90 bytes long, so every
    other row's dwords start on an address that is even but not a multiple of four; a NaN scale byte (255) at the
    start of a row must not leak into the row before through the blocks that do not exist."""
    rng = np.random.default_rng(53)
    N, K = 136, 2880
    sizes = [3, 0, 260, 41]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    total, G = int(offs[-1]), len(sizes)
    (a, pa), (b, pb) = random_operand_any(rng, ea, total, K, 116, 136), random_operand_any(rng, eb, G * N, K, 116, 136)
    # rows 1 and 5 of A and row 1 of every weight start with a NaN block: their own outputs are NaN, no others
    for t in (a, pa):
        t[1][[1, 5], 0] = 255
    for t in (b, pb):
        t[1][1::N, 0] = 255
    da, db = [dev_u8(t) for t in pa], [dev_u8(t) for t in pb]
    out = torch.full((total, N), -7.0, dtype=torch.float32, device="cuda")
    mx.mx_gemm_mbs_elem_grouped(ea, da[0], da[1], da[2], eb, db[0], db[1], db[2], torch.from_numpy(offs).cuda(), N, "f32", out=out)
    got = host(out)
    nan_rows, nan_cols = np.zeros(total, bool), np.zeros(N, bool)
    nan_rows[[1, 5]] = True
    nan_cols[1] = True
    assert np.all(np.isnan(got[nan_rows])) and np.all(np.isnan(got[:, nan_cols]))
    keep = np.ix_(~nan_rows, ~nan_cols)
    assert not np.any(np.isnan(got[keep]))
    for e in range(G):
        lo, hi_ = int(offs[e]), int(offs[e + 1])
        if lo == hi_:
            continue
        rows = np.array([r for r in range(lo, hi_) if not nan_rows[r]])
        a_e = tuple(t[rows] for t in a)
        b_e = tuple(t[e * N:(e + 1) * N][~nan_cols] for t in b)
        assert_gemm_elem_ok(oracle, got[rows][:, ~nan_cols], ea, a_e, eb, b_e, "group %d" % e)


def test_gemm_elem_exact_on_small_integers(mx, oracle):
    """Products that need no alignment (codes for 0, +-0.5, +-1, +-2, 4) add up exactly: any misplaced element,
    scale byte or sigma shows as an integer-sized error."""
    rng = np.random.default_rng(44)
    pool = np.array([0x00, 0x30, 0xB0, 0x38, 0xB8, 0x40, 0xC0, 0x48], np.uint8)  # E4M3
    for M, N, K in ((300, 200, 640), (200, 300, 1536)):
        a = (rng.choice(pool, (M, K)), rng.integers(124, 131, (M, K // 32), dtype=np.uint8), np.zeros((M, K // 128), np.uint8))
        b = (rng.choice(pool, (N, K)), rng.integers(124, 131, (N, K // 32), dtype=np.uint8), np.zeros((N, K // 128), np.uint8))
        got = host(gpu_gemm(mx, "e4m3", a, "e4m3", b))
        assert np.array_equal(got.astype(np.float64), oracle.elem_gemm("e4m3", a, "e4m3", b))
    # MBS words whose sigma is a power of two or 2/3 (m8 = 0, 128): exact up to the rounding of 2/3
    a = (a[0], a[1], rng.choice(np.array([0, 128], np.uint8), (M, K // 128)))
    want = oracle.elem_gemm("e4m3", a, "e4m3", b)
    got = host(gpu_gemm(mx, "e4m3", a, "e4m3", b))
    assert np.max(np.abs(got - want)) <= 1e-5 * np.sqrt(np.mean(want ** 2))


def test_gemm_elem_bf16_output_and_strided_c(mx, oracle):
    rng = np.random.default_rng(43)
    M, N, K = 96, 136, 512
    a, b = random_operand(rng, "e4m3", M, K, 120, 134), random_operand(rng, "e4m3", N, K, 120, 134)
    c32 = gpu_gemm(mx, "e4m3", a, "e4m3", b, "f32")
    c16 = gpu_gemm(mx, "e4m3", a, "e4m3", b, "bf16")
    assert torch.equal(c16, c32.to(torch.bfloat16))
    big = torch.zeros((M, N + 24), dtype=torch.float32, device="cuda")
    gpu_gemm(mx, "e4m3", a, "e4m3", b, "f32", out=big[:, :N])
    assert torch.equal(big[:, :N], c32) and float(big[:, N:].abs().max()) == 0.0
    # rows of C on 8-byte (fp32, bf16) and 4-byte (bf16) boundaries: the epilogue's narrower stores
    for dt, ref, off, pad in ((torch.float32, c32, 2, 26), (torch.bfloat16, c16, 4, 28), (torch.bfloat16, c16, 2, 30)):
        wide = torch.full((M, N + pad), -3.0, dtype=dt, device="cuda")
        gpu_gemm(mx, "e4m3", a, "e4m3", b, "f32" if dt == torch.float32 else "bf16", out=wide[:, off:off + N])
        assert torch.equal(wide[:, off:off + N], ref), (dt, off)
        frame = wide.clone()
        frame[:, off:off + N] = -3.0
        assert bool((frame == -3.0).all()), (dt, off)
    # an odd number of columns and a C that only allows element stores
    odd = torch.zeros((M, N + 3), dtype=torch.bfloat16, device="cuda")
    gpu_gemm(mx, "e4m3", a, "e4m3", (b[0][:N - 1], b[1][:N - 1], b[2][:N - 1]), "bf16", out=odd[:, 1:N])
    assert torch.equal(odd[:, 1:N], c16[:, :N - 1]) and float(odd[:, N:].abs().max()) == 0.0 and float(odd[:, 0].abs().max()) == 0.0


def test_gemm_elem_empty_and_unsupported(mx):
    z = torch.empty((0, 128), dtype=torch.uint8, device="cuda")
    s = torch.empty((0, 4), dtype=torch.uint8, device="cuda")
    b = torch.zeros((8, 128), dtype=torch.uint8, device="cuda")
    bs = torch.full((8, 4), 127, dtype=torch.uint8, device="cuda")
    assert mx.mx_gemm_mbs_elem("e4m3", z, s, None, "e4m3", b, bs, None).shape == (0, 8)
    b64 = torch.zeros((8, 64), dtype=torch.uint8, device="cuda")
    s64 = torch.full((8, 2), 127, dtype=torch.uint8, device="cuda")
    with pytest.raises(mx.MxError) as e:
        mx.mx_gemm_mbs_elem("e4m3", b64, s64, None, "e4m3", b64, s64, None)  # K below one macro block
    assert e.value.status == -4
    b96 = torch.zeros((8, 224), dtype=torch.uint8, device="cuda")
    s96 = torch.full((8, 7), 127, dtype=torch.uint8, device="cuda")
    with pytest.raises(mx.MxError) as e:
        mx.mx_gemm_mbs_elem("e4m3", b96, s96, None, "e4m3", b96, s96, None)  # K % 64 != 0
    assert e.value.status == -4


def test_gemm_elem_quantized_tensors_and_repeat(mx, oracle):
    """Operands quantized on the GPU from heavy-tailed activations and Gaussian weights, every rule; the whole
    result against the oracle, and a second launch bit-identical to the first."""
    from paper_2603_08713_amd import synth

    M, N, K = 200, 300, 1152
    a_bits = synth.activations_student_t(M, K, 3.0, 0.01, 20.0, 3)
    w_bits = synth.gaussian(N, K, 0.02, 4)
    xa, xw = dev_bf16(a_bits), dev_bf16(w_bits)
    for ea, eb, rule in (("e4m3", "e4m3", "oas"), ("e5m2", "e4m3", "floor"), ("e4m3", "e5m2", "ocp")):
        a = mx.mx_quantize_elem(xa, ea, rule)
        b = mx.mx_quantize_elem(xw, eb, rule)
        c = mx.mx_gemm_mbs_elem(ea, a[0], a[1], a[2], eb, b[0], b[1], b[2], "f32")
        c2 = mx.mx_gemm_mbs_elem(ea, a[0], a[1], a[2], eb, b[0], b[1], b[2], "f32")
        torch.cuda.synchronize()
        assert torch.equal(c, c2)
        ah, bh = [host(t) for t in a], [host(t) for t in b]
        oa, ob = oracle.elem_quantize(ea, a_bits, rule, mbs=True), oracle.elem_quantize(eb, w_bits, rule, mbs=True)
        assert all(np.array_equal(x, y) for x, y in zip(ah, oa)) and all(np.array_equal(x, y) for x, y in zip(bh, ob))
        assert_gemm_close(host(c), oracle.elem_gemm(ea, oa, eb, ob), "%s x %s %s" % (ea, eb, rule))


def test_gemm_elem_first_launch_of_a_process_matches_later_ones(mx):
    """A kernel's very first launch in a process runs with cold instruction caches and address translation, so its
    wavefronts drift apart far more than later: a load that the pipeline's waits do not cover would show as a
    wrong patch of C in that launch only.  A fresh process multiplies a large problem in each form of the kernel
    (fast and general, with and without MBS words), each launched for the first time there, and compares with the
    second launch."""
    import os
    import subprocess
    import sys

    code = """
import torch, paper_2603_08713_amd as mx
torch.manual_seed(0)
a = torch.randn(8192, 8192, device="cuda").to(torch.bfloat16)
w = (torch.randn(14336, 8192, device="cuda") * 0.02).to(torch.bfloat16)
qa, qw = mx.mx_quantize_elem(a, "e4m3", "oas"), mx.mx_quantize_elem(w, "e4m3", "oas")
first = mx.mx_gemm_mbs_elem("e4m3", *qa, "e4m3", *qw, "bf16")
again = mx.mx_gemm_mbs_elem("e4m3", *qa, "e4m3", *qw, "bf16")
p1 = mx.mx_gemm_mbs_elem("e4m3", qa[0], qa[1], None, "e4m3", qw[0], qw[1], None, "bf16")
p2 = mx.mx_gemm_mbs_elem("e4m3", qa[0], qa[1], None, "e4m3", qw[0], qw[1], None, "bf16")
torch.cuda.synchronize()
assert torch.equal(first, again), int((first != again).sum())
assert torch.equal(p1, p2), int((p1 != p2).sum())
# general form: K = 7808 = 61 macro blocks
k = 7808
qa, qw = mx.mx_quantize_elem(a[:, :k].contiguous(), "e5m2", "oas"), mx.mx_quantize_elem(w[:, :k].contiguous(), "e4m3", "oas")
for words in (True, False):
    fn = lambda: mx.mx_gemm_mbs_elem("e5m2", qa[0], qa[1], qa[2] if words else None, "e4m3", qw[0], qw[1], qw[2] if words else None, "bf16")
    c1 = fn(); c2 = fn()
    torch.cuda.synchronize()
    assert torch.equal(c1, c2), (words, int((c1 != c2).sum()))
print("first launch ok")
"""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, PYTHONPATH=root + os.pathsep + os.environ.get("PYTHONPATH", ""))
    out = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=280)
    assert out.returncode == 0 and "first launch ok" in out.stdout, out.stdout[-2000:] + out.stderr[-2000:]


def test_gemm_elem_full_size_sampled_rows(mx, oracle):
    """Llama-3-8B FFN up-projection shape in MXFP8 (E4M3), as bench.py launches it: sampled output rows against
    the fp64 oracle, and QSNR(AB) against the bf16 product above MXFP4's (more element bits, same method)."""
    from paper_2603_08713_amd import synth

    M, N, K = 4096, 14336, 4096
    a_bits, w_bits = synth.llama8b_ffn_up(M, N, K)
    xa, xw = dev_bf16(a_bits), dev_bf16(w_bits)
    a = mx.mx_quantize_elem(xa, "e4m3", "oas")
    b = mx.mx_quantize_elem(xw, "e4m3", "oas")
    c = mx.mx_gemm_mbs_elem("e4m3", a[0], a[1], a[2], "e4m3", b[0], b[1], b[2], "f32")
    c16 = mx.mx_gemm_mbs_elem("e4m3", a[0], a[1], a[2], "e4m3", b[0], b[1], b[2], "bf16")
    torch.cuda.synchronize()
    assert torch.equal(c16, c.to(torch.bfloat16))
    assert bool(torch.isfinite(c).all())
    rows = np.sort(np.random.default_rng(9).choice(M, 12, replace=False))
    rows[0], rows[-1] = 0, M - 1
    ah, bh = [host(t) for t in a], [host(t) for t in b]
    want = oracle.elem_gemm("e4m3", ah, "e4m3", bh, rows=rows)
    got = host(c[torch.from_numpy(rows).cuda()])
    assert_gemm_close(got, want, "llama8b e4m3 sampled rows")
    ref = oracle.matmul_bf16(a_bits, w_bits, rows=rows)
    q8 = oracle.qsnr_db(ref, got)
    a4, b4 = mx.mx_quantize_mbs(xa, "oas"), mx.mx_quantize_mbs(xw, "oas")
    c4 = mx.mx_gemm_mbs(a4[0], a4[1], a4[2], b4[0], b4[1], b4[2], "f32")
    q4 = oracle.qsnr_db(ref, host(c4[torch.from_numpy(rows).cuda()]))
    assert q8 > q4 + 10.0, (q8, q4)
