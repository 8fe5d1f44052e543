"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar: bit-exact codes, E8M0 scales and MBS words; GEMM within max|C - C_oracle| <= 1e-3 * RMS(C_oracle)
on the fp32-output kernel; the bf16 output must equal the bf16 rounding of the kernel's own fp32
output (bf16 rounding alone exceeds 1e-3 RMS, so it cannot be held to that bound directly).
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

RULES = ("ocp", "floor", "oas")
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
    return t.cpu().numpy()


def assert_quant_equal(mx, oracle, bits, rule, mbs, what=""):
    x = dev_bf16(bits)
    if mbs:
        c, s, w = mx.mx_quantize_mbs(x, rule)
    elif rule == "oas":
        c, s = mx.mx_quantize_oas(x)
        w = None
    else:
        c, s = mx.mx_quantize(x, rule)
        w = None
    torch.cuda.synchronize()
    oc, os_, ow = oracle.quantize(bits, rule, mbs=mbs)
    tag = "%s rule=%s mbs=%s" % (what, rule, mbs)
    if mbs:
        bad = np.argwhere(host(w) != ow)
        assert bad.size == 0, "%s: %d MBS words differ, first at %s" % (tag, len(bad), bad[:3])
    bad = np.argwhere(host(s) != os_)
    assert bad.size == 0, "%s: %d scales differ, first at %s gpu=%s oracle=%s" % (
        tag, len(bad), bad[:3], host(s)[tuple(bad[0])], os_[tuple(bad[0])])
    bad = np.argwhere(host(c) != oc)
    assert bad.size == 0, "%s: %d code bytes differ, first at %s gpu=%#x oracle=%#x" % (
        tag, len(bad), bad[:3], host(c)[tuple(bad[0])], oc[tuple(bad[0])])



# ------------------------------------------------------------------------------------------------
# quantizers
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("hw", [1, 0])
@pytest.mark.parametrize("mbs", [False, True])
@pytest.mark.parametrize("rule", RULES)
def test_quantize_tiny_config(mx, oracle, rule, mbs, hw):
    from paper_2603_08713_amd import synth

    with mx.forced(quantize_hw=hw):
        a, w = synth.tiny(0)
        assert_quant_equal(mx, oracle, a, rule, mbs, "tiny A")
        assert_quant_equal(mx, oracle, w, rule, mbs, "tiny W")


@pytest.mark.parametrize("hw", [1, 0])
def test_quantize_every_bf16_pattern(mx, oracle, hw):
    """All 65536 bf16 patterns (subnormals, Inf, NaN, both zeros): in natural order (blocks of
    similar magnitude), and shuffled so that blocks mix magnitudes; plus exact ties."""
    with mx.forced(quantize_hw=hw):
        allbits = np.arange(65536, dtype=np.uint16).reshape(128, 512)
        rng = np.random.default_rng(0)
        finite = allbits.reshape(-1)[(allbits.reshape(-1) & 0x7F80) != 0x7F80]
        mid = finite[((finite >> 7) & 0xFF > 100) & ((finite >> 7) & 0xFF < 150)]
        cases = {
            "natural": allbits,
            "shuffled-all": rng.permutation(allbits.reshape(-1)).reshape(128, 512),
            "shuffled-mid": rng.choice(mid, size=(96, 1024)),
            "shuffled-finite": rng.choice(finite, size=(64, 640)),
        }
        # ties: k/4 * 2^e with a block maximum that makes the scale 1, 2 or 1/2
        t = (np.arange(0, 32, dtype=np.float32) / 4.0)[None, :] * np.float32(2.0) ** np.arange(-3, 5, dtype=np.float32)[:, None]
        tb = (t.view(np.uint32) >> 16).astype(np.uint16)
        tb[:, 1::2] |= 0x8000
        cases["ties"] = np.tile(tb, (1, 4))
        for name, bits in cases.items():
            for rule in RULES:
                for mbs in (False, True):
                    assert_quant_equal(mx, oracle, bits, rule, mbs, name)


@pytest.mark.parametrize("rows,K,ld", [(1, 32, 32), (3, 96, 104), (5, 2880, 2880), (2, 4096 + 64, 4232), (7, 512, 512),
                                        (130, 160, 160)])
def test_quantize_ragged_shapes(mx, oracle, rows, K, ld):
    rng = np.random.default_rng(rows * 1000 + K)
    from paper_2603_08713_amd import synth

    full = synth.to_bf16_bits(rng.standard_t(3, (rows, ld)))
    x_full = dev_bf16(full)
    x = x_full[:, :K]
    for rule in ("oas", "ocp"):
        c, s, w = mx.mx_quantize_mbs(x, rule)
        c2, s2 = mx.mx_quantize(x, rule)
        torch.cuda.synchronize()
        oc, os_, ow = oracle.quantize(full[:, :K], rule, mbs=True)
        assert np.array_equal(host(w), ow) and np.array_equal(host(s), os_) and np.array_equal(host(c), oc)
        oc, os_, _ = oracle.quantize(full[:, :K], rule, mbs=False)
        assert np.array_equal(host(s2), os_) and np.array_equal(host(c2), oc)


def test_quantize_empty(mx):
    x = torch.empty((0, 128), dtype=torch.bfloat16, device="cuda")
    c, s, w = mx.mx_quantize_mbs(x)
    assert c.shape == (0, 64) and s.shape == (0, 4) and w.shape == (0, 1)


def test_quantize_full_size_activation(mx, oracle):
    """Llama-3-8B FFN activation shape (4096 x 4096), the launch configuration bench.py times."""
    from paper_2603_08713_amd import synth

    a = synth.activations_student_t(4096, 4096, 4.0, 0.01, 20.0, 1)
    assert_quant_equal(mx, oracle, a, "oas", True, "llama8b A")
    assert_quant_equal(mx, oracle, a, "ocp", False, "llama8b A")


@pytest.mark.parametrize("rows0,rows1,K", [(64, 256, 512), (5, 3, 2880), (1, 130, 160), (0, 7, 1024), (9, 0, 96), (4096, 1000, 4096)])
def test_quantize_pair_equals_two_calls(mx, oracle, rows0, rows1, K):
    """Two tensors in one launch: identical to the oracle (and so to two separate calls), for every rule;
    row counts that leave partial batches at the seam between the tensors."""
    from paper_2603_08713_amd import synth

    b0 = synth.activations_student_t(max(rows0, 1), K, 4.0, 0.01, 20.0, rows0 + 1)[:rows0]
    b1 = synth.gaussian(max(rows1, 1), K, 0.02, rows1 + 2)[:rows1]
    for rule in RULES:
        q0, q1 = mx.mx_quantize_mbs_pair(dev_bf16(b0), dev_bf16(b1), rule)
        torch.cuda.synchronize()
        for bits, got in ((b0, q0), (b1, q1)):
            if bits.shape[0] == 0:
                continue
            rows = None if bits.shape[0] <= 512 else np.arange(0, bits.shape[0], 37)
            want = oracle.quantize(bits if rows is None else bits[rows], rule, mbs=True)
            for g, w_ in zip(got, want):
                g = host(g)
                assert np.array_equal(g if rows is None else g[rows], w_)


# ------------------------------------------------------------------------------------------------
# few-row GEMM with the activations quantized inside the kernel
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,K", [(1, 64, 512), (7, 200, 1024), (16, 4096, 4096), (17, 16 * 300, 2048), (33, 16 * 600, 512),
                                   (64, 1000, 8192), (16, 14336, 4096)])
def test_gemm_quantize_a_fused(mx, oracle, M, N, K):
    """C = Q(A) B^T in one launch: bit-identical to quantize + GEMM through the two entry points, and within
    tolerance of the oracle; every rule, with and without MBS words on either side, padded rows of A."""
    from paper_2603_08713_amd import synth

    lda = K + 64
    full = synth.activations_student_t(M, lda, 4.0, 0.01, 20.0, M * 31 + N)
    a_bits = np.ascontiguousarray(full[:, :K])
    w_bits = synth.gaussian(N, K, 0.02, N + K)
    xa = dev_bf16(full)[:, :K]
    wq = mx.mx_quantize_mbs(dev_bf16(w_bits), "oas")
    ow = tuple(host(t) for t in wq)
    for rule, a_mbs, b_mbs in (("oas", True, True), ("ocp", False, True), ("floor", True, False), ("oas", False, False)):
        bm = wq[2] if b_mbs else None
        for dt in ("f32", "bf16"):
            got = mx.mx_gemm_mbs_quantize_a(xa, rule, wq[0], wq[1], bm, dt, a_use_mbs=a_mbs)
            aq = mx.mx_quantize_mbs(xa, rule) if a_mbs else mx.mx_quantize(xa, rule) + (None,)
            two = mx.mx_gemm_mbs(aq[0], aq[1], aq[2], wq[0], wq[1], bm, dt)
            torch.cuda.synchronize()
            assert torch.equal(got, two), "rule=%s a_mbs=%s b_mbs=%s %s" % (rule, a_mbs, b_mbs, dt)
        rows = None if M * N <= 1 << 16 else np.array([0, M - 1])
        want = oracle.gemm(oracle.quantize(a_bits, rule, mbs=a_mbs), (ow[0], ow[1], ow[2] if b_mbs else None), rows=rows)
        g32 = host(mx.mx_gemm_mbs_quantize_a(xa, rule, wq[0], wq[1], bm, "f32", a_use_mbs=a_mbs))
        g32 = g32 if rows is None else g32[rows]
        assert np.abs(g32 - want).max() <= GEMM_TOL * np.sqrt(np.mean(want ** 2))


def test_gemm_quantize_a_fused_edge_values(mx, oracle):
    """Activation blocks outside the fp32 route's range (subnormal, tiny, huge, zero rows, Inf/NaN): the
    in-kernel quantizer must agree with the quantizer kernel to the bit, which the product shows."""
    rng = np.random.default_rng(41)
    M, N, K = 16, 256, 1024
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[1] *= np.float32(2.0 ** -110)
    x[2] *= np.float32(2.0 ** -130)
    x[3] *= np.float32(2.0 ** 120)
    x[4] = 0
    x[5, 100:140] *= np.float32(2.0 ** -120)
    x[6, ::3] = 0
    bits = (x.view(np.uint32) >> 16).astype(np.uint16)
    bits[7, 5] = 0x7F80       # +Inf
    bits[8, 900] = 0xFFC0     # NaN
    w_bits = (rng.standard_normal((N, K)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    wq = mx.mx_quantize_mbs(dev_bf16(w_bits), "oas")
    xa = dev_bf16(bits)
    for rule in RULES:
        for a_mbs in (True, False):
            got = mx.mx_gemm_mbs_quantize_a(xa, rule, *wq, "f32", a_use_mbs=a_mbs)
            aq = mx.mx_quantize_mbs(xa, rule) if a_mbs else mx.mx_quantize(xa, rule) + (None,)
            two = mx.mx_gemm_mbs(*aq, *wq, "f32")
            torch.cuda.synchronize()
            g, t2 = host(got), host(two)
            assert np.array_equal(np.isnan(g), np.isnan(t2))
            assert not np.isnan(g[:7]).any()
            assert np.array_equal(g[~np.isnan(g)], t2[~np.isnan(t2)]), "rule=%s a_mbs=%s" % (rule, a_mbs)


def test_gemm_first_launch_of_a_process_matches_later_ones(mx):
    """Regression: a kernel's very first launch in a process runs with cold instruction caches and address
    translation, so its wavefronts drift apart far more than later; the prologue of the main kernel once let a
    load of stage 1 slip past the barrier that publishes it, which showed as a wrong patch of C in that first
    launch only.  A fresh process multiplies a large problem twice (with MBS and without) and compares."""
    import os
    import subprocess
    import sys

    code = """
import torch, paper_2603_08713_amd as mx
torch.manual_seed(0)
a = torch.randn(8192, 8192, device="cuda").to(torch.bfloat16)
w = (torch.randn(28672, 8192, device="cuda") * 0.02).to(torch.bfloat16)
qa, qw = mx.mx_quantize_mbs(a, "oas"), mx.mx_quantize_mbs(w, "oas")
first = mx.mx_gemm_mbs(*qa, *qw, "bf16")
again = mx.mx_gemm_mbs(*qa, *qw, "bf16")
p1 = mx.mx_gemm(qa[0], qa[1], qw[0], qw[1], "bf16")
p2 = mx.mx_gemm(qa[0], qa[1], qw[0], qw[1], "bf16")
torch.cuda.synchronize()
assert torch.equal(first, again), int((first != again).sum())
assert torch.equal(p1, p2), int((p1 != p2).sum())
# the other forms of the kernel, each launched for the first time here: 128 x 128 tiles, and the general form
# (K = 2880) plain, with MBS and grouped
for m, n, k in ((2048, 2048, 8192), (8192, 5760, 2880)):
    qa, qw = mx.mx_quantize_mbs(a[:m, :k].contiguous(), "oas"), mx.mx_quantize_mbs(w[:n, :k].contiguous(), "oas")
    for fn in (lambda: mx.mx_gemm_mbs(*qa, *qw, "bf16"), lambda: mx.mx_gemm(qa[0], qa[1], qw[0], qw[1], "bf16")):
        c1 = fn(); c2 = fn()
        torch.cuda.synchronize()
        assert torch.equal(c1, c2), (m, n, k, int((c1 != c2).sum()))
off = torch.tensor([0, 3000, 3000, 8192], dtype=torch.int64, device="cuda")
g1 = mx.mx_gemm_mbs_grouped(*qa, *qw, off, 1920, "bf16"); g2 = mx.mx_gemm_mbs_grouped(*qa, *qw, off, 1920, "bf16")
torch.cuda.synchronize()
assert torch.equal(g1, g2), int((g1 != g2).sum())
print("first launch ok")
"""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    env = dict(os.environ, PYTHONPATH=root + os.pathsep + os.environ.get("PYTHONPATH", ""))
    out = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=280)
    assert out.returncode == 0 and "first launch ok" in out.stdout, out.stdout[-2000:] + out.stderr[-2000:]


@pytest.mark.parametrize("M,N,K", [(4096, 14336, 4096), (2048, 2048, 2048), (3000, 2880, 2880), (700, 530, 2016)])
def test_gemm_repeated_launches_are_bit_identical(mx, M, N, K):
    """The kernels have no atomics and a fixed summation order, so every launch on the same operands must give
    the same bits; a difference means a synchronisation hole (fast form, small tiles, both general forms)."""
    rng = np.random.default_rng(M + N + K)
    a, b = [dev_u8(t) for t in random_operand(rng, M, K, 120, 134)], [dev_u8(t) for t in random_operand(rng, N, K, 120, 134)]
    first_m = mx.mx_gemm_mbs(*a, *b, "bf16")
    first_p = mx.mx_gemm(a[0], a[1], b[0], b[1], "bf16")
    for rep in range(12):
        assert torch.equal(mx.mx_gemm_mbs(*a, *b, "bf16"), first_m), rep
        assert torch.equal(mx.mx_gemm(a[0], a[1], b[0], b[1], "bf16"), first_p), rep


def test_hip_graph_replay_matches_eager(mx, oracle):
    """The entry points launch on the caller's stream, allocate nothing and never synchronise, so a step can be
    captured in a HIP graph.  Every replay (with eager work and synchronisations in between) must reproduce
    the eager result bit for bit: the decode step in both forms and the prefill step."""
    from paper_2603_08713_amd import synth

    a_bits, w_bits = synth.decode_skinny(512, 1024)
    xa, xw = dev_bf16(a_bits), dev_bf16(w_bits)
    wq = mx.mx_quantize_mbs(xw, "oas")
    big_a, big_w = dev_bf16(synth.activations_student_t(300, 1024, 4.0, 0.01, 20.0, 3)), dev_bf16(synth.gaussian(384, 1024, 0.02, 4))
    # eager results (also warms up everything that must not happen during capture)
    aq = mx.mx_quantize_mbs(xa, "oas")
    want_two = mx.mx_gemm_mbs(*aq, *wq, "bf16")
    want_fused = mx.mx_gemm_mbs_quantize_a(xa, "oas", *wq, "bf16")
    pa, pw = mx.mx_quantize_mbs_pair(big_a, big_w, "oas")
    want_big = mx.mx_gemm_mbs(*pa, *pw, "f32")
    torch.cuda.synchronize()
    # static buffers of the captured steps
    aq_g = tuple(torch.zeros_like(t) for t in aq)
    pa_g, pw_g = tuple(torch.zeros_like(t) for t in pa), tuple(torch.zeros_like(t) for t in pw)
    out_two, out_fused, out_big = torch.zeros_like(want_two), torch.zeros_like(want_fused), torch.zeros_like(want_big)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        mx.mx_quantize_mbs(xa, "oas", *aq_g)
        mx.mx_gemm_mbs(*aq_g, *wq, "bf16", out=out_two)
        mx.mx_gemm_mbs_quantize_a(xa, "oas", *wq, "bf16", out=out_fused)
        mx.mx_quantize_mbs_pair(big_a, big_w, "oas", pa_g, pw_g)
        mx.mx_gemm_mbs(*pa_g, *pw_g, "f32", out=out_big)
    for replay in range(4):
        for t in (out_two, out_fused, out_big) + aq_g + pa_g + pw_g:
            t.fill_(1)                                   # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_two, want_two) and torch.equal(out_fused, want_fused), replay
        assert torch.equal(out_big, want_big), replay
        assert all(torch.equal(a, b) for a, b in zip(aq_g, aq))


# ------------------------------------------------------------------------------------------------
# MBS-Dynamic quantizer (searched word)
# ------------------------------------------------------------------------------------------------
def assert_dynamic_valid(mx, oracle, bits, rule="oas", what="", oracle_rows=None, cand_first=0, cand_count=16, cand_stride=16):
    """The kernel sums squared errors in fp32, the oracle (Eq. 6 with the true error) in fp64, so near-ties may
    fall either way: what is unique is compared, the rest is checked for validity.  GPU on all rows; oracle on
    all rows or on the listed ones (rows are independent).
      * the chosen word is the static word or one of the candidates;
      * its exact sum of squared errors is within 1e-5 of the least one on offer, and where the least one is
        separated from the runner-up by more than 1e-4 the word itself is the oracle's;
      * windows the entry point documents as not searched (Inf/NaN inside, absmax outside [2^-63, 2^123)) keep
        the static word;
      * codes and scales are, bit for bit, those of the chosen word."""
    c, s, w = mx.mx_quantize_mbs_dynamic(dev_bf16(bits), rule, cand_first, cand_count, cand_stride)
    torch.cuda.synchronize()
    sel = slice(None) if oracle_rows is None else oracle_rows
    x = np.ascontiguousarray(bits[sel])
    gw, gs, gc = host(w)[sel], host(s)[sel], host(c)[sel]
    tag = "%s rule=%s cands=(%d, %d, %d)" % (what, rule, cand_first, cand_count, cand_stride)
    static = oracle.quantize(x, rule, mbs=True)[2]
    steps = [0] + [(cand_first + j) * cand_stride for j in range(cand_count)]
    cand = np.stack([((static.astype(np.int64) + st) % 256).astype(np.uint8) for st in steps])
    sse = np.stack([oracle.mbs_sse_rows(x, cw, rule) for cw in cand])           # [1 + count, rows, nmac]
    rows, K = x.shape
    nmac = static.shape[1]
    pad = np.zeros((rows, nmac * 128), np.float64)
    val = oracle.bf16_to_f64(x)
    pad[:, :K] = np.where(np.isfinite(val), np.abs(val), 0.0)
    absmax = pad.reshape(rows, nmac, 128).max(2)
    searched = (sse[0] >= 0) & (absmax >= 2.0 ** -63) & (absmax < 2.0 ** 123)
    assert (cand == gw[None]).any(0).all(), "%s: a chosen word is not a candidate" % tag
    bad = np.argwhere(~searched & (gw != static))
    assert bad.size == 0, "%s: %d windows outside the searched domain left the static word, first %s" % (tag, len(bad), bad[:3])
    got = oracle.mbs_sse_rows(x, gw, rule)
    best = sse.min(0)
    bad = np.argwhere(searched & (got > best * (1 + 1e-5)))
    assert bad.size == 0, "%s: %d windows miss the least SSE, first %s got %s best %s" % (
        tag, len(bad), bad[:3], got[tuple(bad[0])], best[tuple(bad[0])])
    _, _, ow = oracle.quantize_mbs_dynamic(x, rule, cand_first, cand_count, cand_stride)
    others = np.where(cand == ow[None], np.inf, sse)                           # every slot that is not the oracle's word
    clear = searched & (others.min(0) > best * (1 + 1e-4))
    bad = np.argwhere(clear & (gw != ow))
    assert bad.size == 0, "%s: %d clearly separated windows differ from the oracle's word, first %s" % (tag, len(bad), bad[:3])
    oc, os_, _ = oracle.quantize_given_mbs(x, gw, rule)
    for name, g, want in (("scales", gs, os_), ("code bytes", gc, oc)):
        bad = np.argwhere(g != want)
        assert bad.size == 0, "%s: %d %s differ from those of the chosen word, first at %s gpu=%s oracle=%s" % (
            tag, len(bad), name, bad[:3], g[tuple(bad[0])], want[tuple(bad[0])])
    return gw, float(clear.mean())


@pytest.mark.parametrize("cands", [dict(), dict(cand_first=-8, cand_count=16, cand_stride=1),
                                   dict(cand_first=-100, cand_count=256, cand_stride=3), dict(cand_count=0),
                                   dict(cand_first=5, cand_count=7, cand_stride=-21)])
def test_quantize_dynamic_small(mx, oracle, cands):
    from paper_2603_08713_amd import synth

    a, w = synth.tiny(0)
    moved = 0
    for rule in RULES:
        for name, bits in (("tiny A", a), ("tiny W", w), ("t(3) outliers", synth.activations_student_t(37, 1024 + 64, 3.0, 0.01, 50.0, 9))):
            words, clear = assert_dynamic_valid(mx, oracle, bits, rule, name, **cands)
            moved += int((words != oracle.quantize(bits, rule, mbs=True)[2]).sum())
            assert clear > 0.5, (name, clear)               # most windows have a clear winner: the word check bites
    assert (moved > 0) == (cands.get("cand_count", 16) > 0)   # the search is really exercised


def test_quantize_dynamic_edge_cases(mx, oracle):
    """Every bf16 pattern (natural order and shuffled: Inf/NaN, subnormals, huge values: windows outside
    the search's domain keep the static word), ties, zero rows, blocks far below their window's absmax,
    and values on the grid beside tiny ones (squared errors in the subnormal range)."""
    rng = np.random.default_rng(21)
    allbits = np.arange(65536, dtype=np.uint16).reshape(128, 512)
    finite = allbits.reshape(-1)[(allbits.reshape(-1) & 0x7F80) != 0x7F80]
    cases = {
        "natural": allbits,
        "shuffled-all": rng.permutation(allbits.reshape(-1)).reshape(128, 512),
        "shuffled-finite": rng.choice(finite, size=(64, 640)),
        "zeros": np.zeros((3, 256), np.uint16),
    }
    spread = np.random.default_rng(22).standard_normal((48, 512)).astype(np.float32)
    for r in range(48):
        spread[r, 32:64] *= np.float32(2.0) ** -(r + 2)        # one block 2..49 binades down
        spread[r, 200:210] *= np.float32(2.0) ** -(2 * r)      # single tiny elements
    cases["spread"] = (spread.view(np.uint32) >> 16).astype(np.uint16)
    grid = np.array([0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0, 0.0], np.float32)
    g = rng.choice(grid, size=(40, 256)) * np.float32(2.0) ** rng.integers(-3, 4, size=(40, 1)).astype(np.float32)
    g[:, 0] = 6.0 * g[:, 1].clip(min=1.0)
    for r in range(40):
        g[r, 17::29] = np.float32(2.0) ** -(60 + r)             # tiny, beside exactly representable values
    cases["grid+tiny"] = (g.view(np.uint32) >> 16).astype(np.uint16)
    for name, bits in cases.items():
        for rule in RULES:
            assert_dynamic_valid(mx, oracle, bits, rule, name)
        assert_dynamic_valid(mx, oracle, bits, "oas", name, cand_first=-128, cand_count=256, cand_stride=1)


@pytest.mark.parametrize("rows,K,ld", [(1, 32, 32), (3, 96, 104), (5, 2880, 2880), (2, 4096 + 64, 4232), (130, 160, 160)])
def test_quantize_dynamic_ragged_shapes(mx, oracle, rows, K, ld):
    from paper_2603_08713_amd import synth

    full = synth.gaussian(rows, ld, 0.02, rows * 7 + K)
    x = dev_bf16(full)[:, :K]
    c, s, w = mx.mx_quantize_mbs_dynamic(x, "oas")
    torch.cuda.synchronize()
    # strided input: same result as the packed copy, which is held to the oracle
    gw, _ = assert_dynamic_valid(mx, oracle, np.ascontiguousarray(full[:, :K]), "oas", "ragged %dx%d" % (rows, K))
    assert np.array_equal(host(w), gw)
    oc, os_, _ = oracle.quantize_given_mbs(np.ascontiguousarray(full[:, :K]), gw, "oas")
    assert np.array_equal(host(s), os_) and np.array_equal(host(c), oc)


def test_quantize_dynamic_full_size_weights_sampled_rows(mx, oracle):
    """The Llama-3-8B FFN up-projection weight (14336 x 4096), every row on the GPU, 512 seeded rows
    on the oracle; and the hybrid GEMM (searched words for W, static for A) on sampled rows."""
    from paper_2603_08713_amd import synth

    a_bits, w_bits = synth.llama8b_ffn_up()
    rows = np.sort(np.random.default_rng(31).choice(w_bits.shape[0], 512, replace=False))
    rows[0], rows[-1] = 0, w_bits.shape[0] - 1
    assert_dynamic_valid(mx, oracle, w_bits, "oas", "L3-8B W", oracle_rows=rows)
    wq = mx.mx_quantize_mbs_dynamic(dev_bf16(w_bits), "oas")
    aq = mx.mx_quantize_mbs(dev_bf16(a_bits), "oas")
    C = mx.mx_gemm_mbs(*aq, *wq, out_dtype="f32")
    torch.cuda.synchronize()
    pick = np.sort(np.random.default_rng(32).choice(a_bits.shape[0], 8, replace=False))
    want = oracle.gemm(oracle.quantize(a_bits[pick], "oas", mbs=True), tuple(host(t) for t in wq))
    got = host(C)[pick]
    assert np.abs(got - want).max() <= GEMM_TOL * np.sqrt(np.mean(want ** 2))


# ------------------------------------------------------------------------------------------------
# MBS-Dynamic through the table of Eq. 5
# ------------------------------------------------------------------------------------------------
def golden_lut():
    import os

    lut = np.zeros((2, 64, 16), np.uint16)
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "mbs_lut_fp16.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        lut[int(f[0]), int(f[1])] = [int(h, 16) for h in f[2:]]
    return lut


def test_mbs_lut_build_is_the_oracle_table(mx, oracle):
    """The library builds the table of Eq. 5 itself (fp64, one rounding to fp16): every one of the 2048 entries
    equals the stored table that the oracle wrote."""
    lut = mx.mx_mbs_lut_build()
    torch.cuda.synchronize()
    got = host(lut).view(np.uint16)
    want = golden_lut()
    assert np.array_equal(want, oracle.mbs_lut())
    bad = np.argwhere(got != want)
    assert bad.size == 0, "%d entries differ, first at %s gpu=%#x oracle=%#x" % (len(bad), bad[:3], got[tuple(bad[0])], want[tuple(bad[0])])


def assert_lut_valid(mx, oracle, bits, rule="oas", keep_static=True, what="", oracle_rows=None):
    """The kernel sums Eq. 6 in fp32 (and, for keep_static, the two true errors in fp32), the oracle in fp64: near-ties
    may fall either way, so what is unique is compared and the rest checked for validity.
      * a searched window's word is 16 j or (keep_static) the static word; others keep the static word;
      * the tabulated cost of a picked 16 j is within 1e-4 of the least one; where the least one is separated by more
        than 1e-3 (and, with keep_static, the true errors of the two contenders by more than 1e-4) the word is the oracle's;
      * keep_static: the kept word's true error is not larger than the other contender's by more than 1e-5;
      * codes and scales are, bit for bit, those of the chosen word."""
    lut = golden_lut()
    dlut = torch.from_numpy(lut.view(np.int16)).cuda()
    c, s, w = mx.mx_quantize_mbs_dynamic_lut(dev_bf16(bits), dlut, rule, keep_static)
    torch.cuda.synchronize()
    sel = slice(None) if oracle_rows is None else oracle_rows
    x = np.ascontiguousarray(bits[sel])
    gw, gs, gc = host(w)[sel], host(s)[sel], host(c)[sel]
    tag = "%s rule=%s keep_static=%s" % (what, rule, keep_static)
    rows, K = x.shape
    static = oracle.quantize(x, rule, mbs=True)[2]
    nmac = static.shape[1]
    pad = np.zeros((rows, nmac * 128), np.float64)
    val = oracle.bf16_to_f64(x)
    finite = np.ones((rows, nmac * 128), bool)
    finite[:, :K] = np.isfinite(val)
    pad[:, :K] = np.where(np.isfinite(val), np.abs(val), 0.0)
    absmax = pad.reshape(rows, nmac, 128).max(2)
    searched = finite.reshape(rows, nmac, 128).all(2) & (absmax >= 2.0 ** -63) & (absmax < 2.0 ** 123)
    bad = np.argwhere(~searched & (gw != static))
    assert bad.size == 0, "%s: %d windows outside the searched domain left the static word, first %s" % (tag, len(bad), bad[:3])
    # tabulated costs of all 16 candidates, per window
    cost = np.full((16, rows, nmac), np.inf)
    for r in range(rows):
        for g in range(nmac):
            if searched[r, g]:
                seg = x[r, 128 * g:min(128 * g + 128, K)]
                cost[:, r, g] = [oracle.mbs_lut_cost(seg, j, lut, rule) for j in range(16)]
    jbest = cost.argmin(0)
    least = cost.min(0)
    picked = (gw % 16 == 0) & (cost[(gw // 16).clip(0, 15), np.arange(rows)[:, None], np.arange(nmac)[None, :]] <= least * (1 + 1e-4))
    ok = picked | (gw == static) if keep_static else picked
    bad = np.argwhere(searched & ~ok)
    assert bad.size == 0, "%s: %d windows hold a word that is neither a least-cost candidate nor allowed, first %s word %s" % (
        tag, len(bad), bad[:3], gw[tuple(bad[0])] if len(bad) else None)
    _, _, ow = oracle.quantize_mbs_dynamic_lut(x, lut, rule, keep_static)
    runner = np.sort(cost, axis=0)[1]
    clear = searched & (runner > least * (1 + 1e-3))
    if keep_static:
        w16 = (16 * jbest).astype(np.uint8)
        sse_pick, sse_stat = oracle.mbs_sse_rows(x, np.where(searched, w16, static), rule), oracle.mbs_sse_rows(x, static, rule)
        got_sse = oracle.mbs_sse_rows(x, gw, rule)
        bad = np.argwhere(clear & (got_sse > np.minimum(sse_pick, sse_stat) * (1 + 1e-5)))
        assert bad.size == 0, "%s: %d windows kept the worse of static and picked word, first %s" % (tag, len(bad), bad[:3])
        clear &= np.abs(sse_pick - sse_stat) > 1e-4 * np.maximum(sse_pick, sse_stat)
    bad = np.argwhere(clear & (gw != ow))
    assert bad.size == 0, "%s: %d clearly decided windows differ from the oracle's word, first %s gpu %s oracle %s" % (
        tag, len(bad), bad[:3], gw[tuple(bad[0])] if len(bad) else None, ow[tuple(bad[0])] if len(bad) else None)
    oc, os_, _ = oracle.quantize_given_mbs(x, gw, rule)
    for name, g, want in (("scales", gs, os_), ("code bytes", gc, oc)):
        bad = np.argwhere(g != want)
        assert bad.size == 0, "%s: %d %s differ from those of the chosen word, first at %s" % (tag, len(bad), name, bad[:3])
    return gw, float(clear.mean())


@pytest.mark.parametrize("keep_static", [True, False])
def test_quantize_dynamic_lut_small(mx, oracle, keep_static):
    from paper_2603_08713_amd import synth

    a, w = synth.tiny(0)
    for rule in RULES:
        for name, bits in (("tiny A", a), ("tiny W", w), ("t(3) outliers", synth.activations_student_t(21, 1024 + 64, 3.0, 0.01, 50.0, 9))):
            words, clear = assert_lut_valid(mx, oracle, bits, rule, keep_static, name)
            assert clear > 0.5, (name, clear)                    # most windows are clearly decided: the word check bites
            if rule == "oas":   # (the table knows no saturation: under the other rules the static word mostly stays)
                assert (words != oracle.quantize(bits, rule, mbs=True)[2]).mean() > 0.3   # the search moves words


def test_quantize_dynamic_lut_edge_cases(mx, oracle):
    """Every bf16 pattern (Inf/NaN, subnormals, huge values: windows outside the search's domain keep the static
    word), zero rows, blocks far below their window's absmax, ragged K and strided input."""
    rng = np.random.default_rng(41)
    allbits = np.arange(65536, dtype=np.uint16).reshape(128, 512)
    finite = allbits.reshape(-1)[(allbits.reshape(-1) & 0x7F80) != 0x7F80]
    spread = np.random.default_rng(42).standard_normal((24, 512)).astype(np.float32)
    for r in range(24):
        spread[r, 32:64] *= np.float32(2.0) ** -(2 * r + 2)
        spread[r, 200:210] *= np.float32(2.0) ** -(4 * r)
    cases = {
        "natural": allbits[::4],
        "shuffled-all": rng.permutation(allbits.reshape(-1)).reshape(128, 512)[:32],
        "shuffled-finite": rng.choice(finite, size=(24, 640)),
        "zeros": np.zeros((3, 256), np.uint16),
        "spread": (spread.view(np.uint32) >> 16).astype(np.uint16),
    }
    for name, bits in cases.items():
        assert_lut_valid(mx, oracle, bits, "oas", True, name)
    from paper_2603_08713_amd import synth

    full = synth.gaussian(5, 2880 + 40, 0.02, 77)
    x = dev_bf16(full)[:, :2880]
    lut = torch.from_numpy(golden_lut().view(np.int16)).cuda()
    c, s, w = mx.mx_quantize_mbs_dynamic_lut(x, lut, "oas")
    gw, _ = assert_lut_valid(mx, oracle, np.ascontiguousarray(full[:, :2880]), "oas", True, "ragged 5x2880")
    assert np.array_equal(host(w), gw)


def test_quantize_dynamic_lut_full_size_weights(mx, oracle):
    """The Llama-3-8B FFN up-projection weight, every row on the GPU with the table the library builds, 64 seeded rows
    on the oracle; QSNR against the static words and the exact search."""
    from paper_2603_08713_amd import synth

    _, w_bits = synth.llama8b_ffn_up()
    rows = np.sort(np.random.default_rng(43).choice(w_bits.shape[0], 64, replace=False))
    rows[0], rows[-1] = 0, w_bits.shape[0] - 1
    assert_lut_valid(mx, oracle, w_bits, "oas", True, "L3-8B W", oracle_rows=rows)
    xw = dev_bf16(w_bits[:512])
    ref = xw.to(torch.float64)

    def qsnr(q):
        back = mx.mx_dequantize(q[0], q[1], q[2], "f32").to(torch.float64)
        return float(10.0 * torch.log10((ref * ref).sum() / ((ref - back) ** 2).sum()))

    lut = mx.mx_mbs_lut_build()
    st, lu, ex = qsnr(mx.mx_quantize_mbs(xw, "oas")), qsnr(mx.mx_quantize_mbs_dynamic_lut(xw, lut, "oas")), qsnr(mx.mx_quantize_mbs_dynamic(xw, "oas"))
    assert lu - st > 0.3 and abs(ex - lu) < 0.05, (st, lu, ex)


# ------------------------------------------------------------------------------------------------
# dequantizer and QSNR from both paths
# ------------------------------------------------------------------------------------------------
def test_dequantize_matches_oracle(mx, oracle):
    rng = np.random.default_rng(5)
    rows, K = 37, 2880
    codes = rng.integers(0, 256, (rows, K // 2), dtype=np.uint8)
    scales = rng.integers(100, 150, (rows, K // 32), dtype=np.uint8)
    scales[3, 5] = 255                      # NaN block
    scales[4, 0], scales[4, 1] = 10, 250    # far ends of the normal fp32 range
    words = rng.integers(0, 256, (rows, (K + 127) // 128), dtype=np.uint8)
    for w in (None, words):
        sc = scales.copy()
        if w is None:
            sc[5, 0], sc[5, 1] = 0, 254     # 2^-127 (subnormal results) and overflow to Inf
        want = oracle.dequantize(codes, sc, w)
        with np.errstate(over="ignore"):
            want32 = want.astype(np.float32)
        nan = np.isnan(want32)
        assert nan.sum() == 32
        got32 = host(mx.mx_dequantize(dev_u8(codes), dev_u8(sc), dev_u8(w), "f32"))
        assert np.array_equal(got32[~nan].view(np.uint32), want32[~nan].view(np.uint32))
        assert np.all(np.isnan(got32[nan]))
        got16 = mx.mx_dequantize(dev_u8(codes), dev_u8(sc), dev_u8(w), "bf16").cpu()
        want16 = torch.from_numpy(want32).to(torch.bfloat16)
        assert np.array_equal(got16.view(torch.int16).numpy()[~nan], want16.view(torch.int16).numpy()[~nan])
        assert np.all(np.isnan(got16.float().numpy()[nan]))
    # strided output
    big = torch.zeros((rows, K + 8), dtype=torch.float32, device="cuda")
    mx.mx_dequantize(dev_u8(codes), dev_u8(scales), dev_u8(words), "f32", out=big[:, :K])
    assert float(big[:, K:].abs().max()) == 0.0
    assert torch.equal(torch.nan_to_num(big[:, :K]), torch.nan_to_num(mx.mx_dequantize(dev_u8(codes), dev_u8(scales), dev_u8(words), "f32")))


def test_dequantize_every_scale_byte_and_word(mx, oracle):
    """Every E8M0 byte (0..254 and the NaN code) against every code, and every MBS word: both routes of the
    kernel (two quotients per lane for normal results, element by element at the ends of the range)."""
    rng = np.random.default_rng(6)
    rows, K = 256, 1024 + 32
    codes = rng.integers(0, 256, (rows, K // 2), dtype=np.uint8)
    codes[:, :8] = np.arange(8, dtype=np.uint8) * 0x11 + np.array([0, 0x80, 0x08, 0x88, 0, 0x80, 0x08, 0x88], np.uint8)
    scales = np.repeat(np.arange(rows, dtype=np.uint8)[:, None], K // 32, 1)      # row r: byte r everywhere
    scales[:, 1::3] = rng.integers(0, 255, scales[:, 1::3].shape, dtype=np.uint8)   # mixed bytes inside a wavefront
    words = rng.integers(0, 256, (rows, (K + 127) // 128), dtype=np.uint8)
    words[:, 0] = np.arange(rows, dtype=np.uint8)
    for w in (None, words):
        want = oracle.dequantize(codes, scales, w)
        with np.errstate(over="ignore"):
            want32 = want.astype(np.float32)
        nan = np.isnan(want32)
        got32 = host(mx.mx_dequantize(dev_u8(codes), dev_u8(scales), dev_u8(w), "f32"))
        assert np.array_equal(np.isnan(got32), nan)
        bad = np.argwhere(got32[~nan].view(np.uint32) != want32[~nan].view(np.uint32))
        assert bad.size == 0, "%d fp32 values differ" % len(bad)
        got16 = mx.mx_dequantize(dev_u8(codes), dev_u8(scales), dev_u8(w), "bf16").cpu()
        want16 = torch.from_numpy(want32).to(torch.bfloat16)
        assert np.array_equal(got16.view(torch.int16).numpy()[~nan], want16.view(torch.int16).numpy()[~nan])
        assert np.all(np.isnan(got16.float().numpy()[nan]))


def test_qsnr_identical_from_both_paths(mx, oracle):
    from paper_2603_08713_amd import synth

    a, _ = synth.tiny(0)
    ref = oracle.bf16_to_f64(a)
    ladder = {"plain": ("ocp", False), "+oas": ("oas", False), "+mbs": ("floor", True), "+oas+mbs": ("oas", True)}
    got = {}
    for name, (rule, mbs) in ladder.items():
        oc, os_, ow = oracle.quantize(a, rule, mbs=mbs)
        q_or = oracle.qsnr_db(ref, oracle.dequantize(oc, os_, ow))
        x = dev_bf16(a)
        if mbs:
            c, s, w = mx.mx_quantize_mbs(x, rule)
        else:
            c, s = mx.mx_quantize(x, rule)
            w = None
        xh = host(mx.mx_dequantize(c, s, w, "f32")).astype(np.float64)
        q_gpu = oracle.qsnr_db(ref, xh)
        assert abs(q_or - q_gpu) < 1e-4, (name, q_or, q_gpu)   # fp32 vs fp64 dequantized values
        got[name] = q_gpu
    assert got["+oas"] > got["plain"] and got["+oas+mbs"] > got["+oas"]


# ------------------------------------------------------------------------------------------------
# GEMM
# ------------------------------------------------------------------------------------------------
def quantized(oracle, bits, rule="oas", mbs=True):
    return oracle.quantize(bits, rule, mbs=mbs)


def gpu_gemm(mx, a, b, out_dtype="f32", plain=False):
    da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
    if plain:
        return mx.mx_gemm(da[0], da[1], db[0], db[1], out_dtype)
    return mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], db[2], out_dtype)


def assert_gemm_close(got, want, what=""):
    rms = float(np.sqrt(np.mean(want ** 2)))
    err = float(np.max(np.abs(got.astype(np.float64) - want)))
    assert err <= GEMM_TOL * rms, "%s: max err %.3e vs %.3e (rms %.3e)" % (what, err, GEMM_TOL * rms, rms)


def test_gemm_tiny_config(mx, oracle):
    from paper_2603_08713_amd import synth

    a_bits, w_bits = synth.tiny(0)
    for rule, mbs in (("oas", True), ("ocp", False), ("floor", True)):
        a, b = quantized(oracle, a_bits, rule, mbs), quantized(oracle, w_bits, rule, mbs)
        want = oracle.gemm(a, b)
        got = host(gpu_gemm(mx, a, b, "f32", plain=not mbs))
        assert_gemm_close(got, want, "tiny %s mbs=%s" % (rule, mbs))
    # one-sided MBS and the MBS entry point without any words
    a, b = quantized(oracle, a_bits, "oas", True), quantized(oracle, w_bits, "oas", False)
    assert_gemm_close(host(gpu_gemm(mx, a, b)), oracle.gemm(a, b), "A-only MBS")
    assert_gemm_close(host(gpu_gemm(mx, b, a)), oracle.gemm(b, a), "B-only MBS")
    a = quantized(oracle, a_bits, "oas", False)
    assert_gemm_close(host(gpu_gemm(mx, a, b)), oracle.gemm(a, b), "no words")


def test_gemm_random_codes_and_scales(mx, oracle):
    """Uniformly random codes, a wide spread of E8M0 bytes and random MBS words: exercises every
    nibble, scale byte and lane position of the instruction's operand layout."""
    rng = np.random.default_rng(42)
    for (M, N, K) in ((16, 16, 128), (64, 48, 256), (130, 200, 384), (257, 129, 2880)):
        a = (rng.integers(0, 256, (M, K // 2), dtype=np.uint8), rng.integers(110, 140, (M, K // 32), dtype=np.uint8),
             rng.integers(0, 256, (M, (K + 127) // 128), dtype=np.uint8))
        b = (rng.integers(0, 256, (N, K // 2), dtype=np.uint8), rng.integers(110, 140, (N, K // 32), dtype=np.uint8),
             rng.integers(0, 256, (N, (K + 127) // 128), dtype=np.uint8))
        assert_gemm_close(host(gpu_gemm(mx, a, b)), oracle.gemm(a, b), "mbs %dx%dx%d" % (M, N, K))
        assert_gemm_close(host(gpu_gemm(mx, a, b, plain=True)), oracle.gemm((a[0], a[1], None), (b[0], b[1], None)),
                          "plain %dx%dx%d" % (M, N, K))


def test_gemm_bf16_output_is_rounded_fp32_output(mx, oracle):
    rng = np.random.default_rng(43)
    M, N, K = 96, 136, 512
    a = (rng.integers(0, 256, (M, K // 2), dtype=np.uint8), rng.integers(120, 134, (M, K // 32), dtype=np.uint8),
         rng.integers(0, 256, (M, K // 128), dtype=np.uint8))
    b = (rng.integers(0, 256, (N, K // 2), dtype=np.uint8), rng.integers(120, 134, (N, K // 32), dtype=np.uint8),
         rng.integers(0, 256, (N, K // 128), dtype=np.uint8))
    c32 = gpu_gemm(mx, a, b, "f32")
    c16 = gpu_gemm(mx, a, b, "bf16")
    assert torch.equal(c16, c32.to(torch.bfloat16))
    # strided C
    big = torch.zeros((M, N + 24), dtype=torch.float32, device="cuda")
    da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
    mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], db[2], "f32", out=big[:, :N])
    assert torch.equal(big[:, :N], c32) and float(big[:, N:].abs().max()) == 0.0


def test_gemm_empty_and_zero_k(mx):
    z = torch.empty((0, 64), dtype=torch.uint8, device="cuda")
    s = torch.empty((0, 4), dtype=torch.uint8, device="cuda")
    b = torch.zeros((8, 64), dtype=torch.uint8, device="cuda")
    bs = torch.full((8, 4), 127, dtype=torch.uint8, device="cuda")
    assert mx.mx_gemm(z, s, b, bs).shape == (0, 8)
    # K = 0: an empty sum, C = 0 (every load of the kernel is out of range and reads zero)
    a0, s0 = torch.empty((5, 0), dtype=torch.uint8, device="cuda"), torch.empty((5, 0), dtype=torch.uint8, device="cuda")
    b0, t0 = torch.empty((130, 0), dtype=torch.uint8, device="cuda"), torch.empty((130, 0), dtype=torch.uint8, device="cuda")
    for dt in ("f32", "bf16"):
        out = torch.full((5, 130), 7.0, dtype=torch.float32 if dt == "f32" else torch.bfloat16, device="cuda")
        mx.mx_gemm(a0, s0, b0, t0, dt, out=out)
        assert float(out.abs().max()) == 0.0
        out.fill_(7.0)
        mx.mx_gemm_mbs(a0, s0, s0, b0, t0, t0, dt, out=out)
        assert float(out.abs().max()) == 0.0


def fragment_rows(M, seed):
    """One output row out of every 32-row fragment (every wavefront's every fragment of every tile-row is hit), at a
    seeded offset; first and last row of the matrix included."""
    rows = np.arange(0, M, 32) + np.random.default_rng(seed).integers(0, 32, size=(M + 31) // 32)
    rows = np.minimum(rows, M - 1)
    rows[0], rows[-1] = 0, M - 1
    return rows.astype(np.int64)


def test_gemm_full_size_sampled_rows(mx, oracle):
    """Llama-3-8B FFN up-projection shape; one output row of every 32-row fragment (128 rows, all columns) is
    checked against the fp64 oracle, all rows against cheap invariants."""
    from paper_2603_08713_amd import synth

    M, N, K = 4096, 14336, 4096
    a_bits, w_bits = synth.llama8b_ffn_up(M, N, K)
    xa, xw = dev_bf16(a_bits), dev_bf16(w_bits)
    a = mx.mx_quantize_mbs(xa, "oas")
    b = mx.mx_quantize_mbs(xw, "oas")
    c = mx.mx_gemm_mbs(a[0], a[1], a[2], b[0], b[1], b[2], "f32")
    c16 = mx.mx_gemm_mbs(a[0], a[1], a[2], b[0], b[1], b[2], "bf16")
    torch.cuda.synchronize()
    assert torch.equal(c16, c.to(torch.bfloat16))
    assert bool(torch.isfinite(c).all())
    rows = fragment_rows(M, 9)
    ah, bh = [host(t) for t in a], [host(t) for t in b]
    want = oracle.gemm(ah, bh, rows=rows)
    got = host(c[torch.from_numpy(rows).cuda()])
    assert_gemm_close(got, want, "llama8b sampled rows")
    # the quantized operands themselves are bit-exact at this size
    oa = oracle.quantize(a_bits, "oas", mbs=True)
    assert all(np.array_equal(x, y) for x, y in zip(ah, oa))


def random_operand(rng, rows, K, lo=110, hi=140):
    return (rng.integers(0, 256, (rows, K // 2), dtype=np.uint8), rng.integers(lo, hi, (rows, K // 32), dtype=np.uint8),
            rng.integers(0, 256, (rows, (K + 127) // 128), dtype=np.uint8))


@pytest.mark.parametrize("shape", [2, 3, 4, 6, 7, 8, 9, 10])
def test_gemm_every_tile_shape(mx, oracle, shape):
    """Each kernel forced in turn (2, 6, 7: the fast form without MBS on 256 x 256, 256 x 128 and 128 x 128 tiles;
    3, 4: the fast form with MBS on 256 x 128 and 128 x 128 tiles; 8, 9: the general form with 2-byte pieces on
    256 x 128 and 128 x 128 tiles, 10: the general form with single bytes; these three with and without MBS,
    also on a K that ends in half a stage and on one of a single pair of blocks, and 10 on K % 64 = 32) on sizes
    with ragged tiles in M and N, several K stages, both output types and rows of C that vector stores cannot
    serve."""
    rng = np.random.default_rng(50 + shape)
    with mx.forced(gemm_shape=shape):
        sizes = ((700, 530, 1536), (257, 300, 512)) + (((300, 260, 2880), (130, 129, 64)) if shape in (8, 9, 10) else ())
        sizes += ((200, 140, 2016), (33, 50, 32)) if shape == 10 else ()
        # (the 256 x 128 MBS kernel takes two groups of four stages per loop turn: a K with no such turn and one
        # with a turn followed by a single group, beside the 1536 above, which has exactly one turn)
        sizes += ((300, 200, 1024), (260, 130, 2048)) if shape == 3 else ()
        for (M, N, K) in sizes:
            a, b = random_operand(rng, M, K), random_operand(rng, N, K)
            da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
            for plain in ((True, False) if shape in (8, 9, 10) else (shape in (2, 6, 7),)):
                want = oracle.gemm((a[0], a[1], None), (b[0], b[1], None)) if plain else oracle.gemm(a, b)
                what = "%s shape %d %dx%dx%d" % ("plain" if plain else "mbs", shape, M, N, K)
                c32 = gpu_gemm(mx, a, b, "f32", plain=plain)
                assert_gemm_close(host(c32), want, what)
                assert torch.equal(gpu_gemm(mx, a, b, "bf16", plain=plain), c32.to(torch.bfloat16)), what
                # rows of C that start at odd element offsets: no vector stores, the frame around C stays untouched
                for dt in (torch.float32, torch.bfloat16):
                    big = torch.full((M + 2, N + 3), -3.0, dtype=dt, device="cuda")
                    out, name = big[1:M + 1, 1:N + 1], "f32" if dt == torch.float32 else "bf16"
                    if plain:
                        mx.mx_gemm(da[0], da[1], db[0], db[1], name, out=out)
                    else:
                        mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], db[2], name, out=out)
                    assert torch.equal(out, c32.to(dt)), what
                    frame = big.clone()
                    frame[1:M + 1, 1:N + 1] = -3.0
                    assert bool((frame == -3.0).all()), what
            if shape in (3, 4, 8, 9, 10):  # one-sided MBS: a null array means sigma = 1
                want = oracle.gemm(a, (b[0], b[1], None))
                got = mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], None, "f32")
                assert_gemm_close(host(got), want, "A-only mbs shape %d" % shape)
                want = oracle.gemm((a[0], a[1], None), b)
                got = mx.mx_gemm_mbs(da[0], da[1], None, db[0], db[1], db[2], "f32")
                assert_gemm_close(host(got), want, "B-only mbs shape %d" % shape)


@pytest.mark.parametrize("shape", [2, 3, 8])
def test_gemm_rows_of_c_on_8_byte_boundaries(mx, oracle, shape):
    """Rows of C that start on 8-byte but not on 16-byte boundaries (the epilogue's 8-byte stores), with N a multiple
    of the store width and not: equal to the contiguous result, the frame around C untouched."""
    rng = np.random.default_rng(60 + shape)
    plain = shape == 2
    with mx.forced(gemm_shape=shape):
        for (M, N, K) in ((300, 264, 512), (130, 263, 1024)):
            a, b = random_operand(rng, M, K), random_operand(rng, N, K)
            da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
            c32 = gpu_gemm(mx, a, b, "f32", plain=plain)
            assert_gemm_close(host(c32), oracle.gemm((a[0], a[1], None), (b[0], b[1], None)) if plain else oracle.gemm(a, b),
                              "shape %d %dx%dx%d" % (shape, M, N, K))
            # (row pitch and first element at 8 mod 16 bytes; for bf16 also at 4 mod 8: two elements per store)
            for dt, name, off, mod in ((torch.bfloat16, "bf16", 4, 16), (torch.bfloat16, "bf16", 2, 8), (torch.float32, "f32", 2, 16)):
                width = (N + 7) // 8 * 8 + 3 * off
                big = torch.full((M + 1, width), -3.0, dtype=dt, device="cuda")
                out = big[:M, off:off + N]
                assert out.data_ptr() % mod == mod // 2 and (width * out.element_size()) % mod == mod // 2
                if plain:
                    mx.mx_gemm(da[0], da[1], db[0], db[1], name, out=out)
                else:
                    mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], db[2], name, out=out)
                assert torch.equal(out, c32.to(dt)), (shape, M, N, K, name)
                frame = big.clone()
                frame[:M, off:off + N] = -3.0
                assert bool((frame == -3.0).all()), (shape, M, N, K, name)


def test_gemm_plain_full_size_sampled_rows(mx, oracle):
    """The plain GEMM at the Llama-3-8B FFN shape (it takes the 256 x 256 kernel there): one row of every 32-row
    fragment against the oracle, bf16 output equal to the rounded fp32 output."""
    rng = np.random.default_rng(51)
    M, N, K = 4096, 14336, 4096
    a, b = random_operand(rng, M, K, 120, 134), random_operand(rng, N, K, 120, 134)
    da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
    c = mx.mx_gemm(da[0], da[1], db[0], db[1], "f32")
    c16 = mx.mx_gemm(da[0], da[1], db[0], db[1], "bf16")
    assert torch.equal(c16, c.to(torch.bfloat16))
    rows = fragment_rows(M, 52)
    want = oracle.gemm((a[0], a[1], None), (b[0], b[1], None), rows=rows)
    assert_gemm_close(host(c[torch.from_numpy(rows).cuda()]), want, "plain llama8b sampled rows")


def test_grouped_gemm(mx, oracle):
    rng = np.random.default_rng(77)
    G, N, K = 5, 160, 2880
    counts = np.array([130, 0, 17, 256, 1])
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    M = int(offsets[-1])
    a = (rng.integers(0, 256, (M, K // 2), dtype=np.uint8), rng.integers(118, 136, (M, K // 32), dtype=np.uint8),
         rng.integers(0, 256, (M, (K + 127) // 128), dtype=np.uint8))
    b = (rng.integers(0, 256, (G * N, K // 2), dtype=np.uint8), rng.integers(118, 136, (G * N, K // 32), dtype=np.uint8),
         rng.integers(0, 256, (G * N, (K + 127) // 128), dtype=np.uint8))
    da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
    out = torch.full((M + 3, N), -7.0, dtype=torch.float32, device="cuda")
    mx.mx_gemm_mbs_grouped(da[0], da[1], da[2], db[0], db[1], db[2], torch.from_numpy(offsets).cuda(), N, "f32",
                           out=out[:M])
    got = host(out)
    assert np.all(got[M:] == -7.0)
    for e in range(G):
        lo, hi = offsets[e], offsets[e + 1]
        if lo == hi:
            continue
        want = oracle.gemm(tuple(t[lo:hi] for t in a), tuple(t[e * N:(e + 1) * N] for t in b))
        assert_gemm_close(got[lo:hi], want, "group %d" % e)


def test_grouped_gemm_many_groups(mx, oracle):
    """More groups than a wavefront has lanes (the kernel looks its group up 64 groups at a time), with empty groups
    at the start, across the boundary between the two passes and at the end, and groups of more than one tile-row."""
    rng = np.random.default_rng(78)
    G, N, K = 70, 96, 256
    counts = rng.integers(1, 40, G)
    counts[[0, 1, 62, 63, 64, 65, 69]] = 0
    counts[5], counts[66] = 300, 130
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    M = int(offsets[-1])
    a, b = random_operand(rng, M, K, 118, 136), random_operand(rng, G * N, K, 118, 136)
    da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
    doff = torch.from_numpy(offsets).cuda()
    out = torch.full((M + 3, N), -7.0, dtype=torch.float32, device="cuda")
    mx.mx_gemm_mbs_grouped(da[0], da[1], da[2], db[0], db[1], db[2], doff, N, "f32", out=out[:M])
    plain = mx.mx_gemm_mbs_grouped(da[0], da[1], None, db[0], db[1], None, doff, N, "f32")
    got, got_plain = host(out), host(plain)
    assert np.all(got[M:] == -7.0)
    for e in range(G):
        lo, hi = offsets[e], offsets[e + 1]
        if lo == hi:
            continue
        rows_a, rows_b = tuple(t[lo:hi] for t in a), tuple(t[e * N:(e + 1) * N] for t in b)
        assert_gemm_close(got[lo:hi], oracle.gemm(rows_a, rows_b), "group %d of %d" % (e, G))
        assert_gemm_close(got_plain[lo:hi], oracle.gemm((rows_a[0], rows_a[1], None), (rows_b[0], rows_b[1], None)),
                          "group %d of %d, no words" % (e, G))


@pytest.mark.parametrize("M", [1, 7, 16, 17, 33, 64])
def test_gemm_few_rows(mx, oracle, M):
    """The few-row (decode) kernel: every fragment count, ragged N, K of one to several load groups per
    wavefront, plain / one-sided / two-sided MBS, both output types."""
    rng = np.random.default_rng(90 + M)
    for (N, K) in ((1000, 512), (48, 1536), (530, 8192)):
        a, b = random_operand(rng, M, K), random_operand(rng, N, K)
        da, db = [dev_u8(t) for t in a], [dev_u8(t) for t in b]
        c32 = mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], db[2], "f32")
        assert_gemm_close(host(c32), oracle.gemm(a, b), "few rows mbs %dx%dx%d" % (M, N, K))
        assert torch.equal(mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], db[2], "bf16"), c32.to(torch.bfloat16))
        assert_gemm_close(host(mx.mx_gemm(da[0], da[1], db[0], db[1], "f32")),
                          oracle.gemm((a[0], a[1], None), (b[0], b[1], None)), "few rows plain %dx%dx%d" % (M, N, K))
        assert_gemm_close(host(mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], None, "f32")),
                          oracle.gemm(a, (b[0], b[1], None)), "few rows A-only %dx%dx%d" % (M, N, K))
        assert_gemm_close(host(mx.mx_gemm_mbs(da[0], da[1], None, db[0], db[1], db[2], "f32")),
                          oracle.gemm((a[0], a[1], None), b), "few rows B-only %dx%dx%d" % (M, N, K))
        big = torch.full((M + 2, N + 3), -3.0, dtype=torch.float32, device="cuda")
        mx.mx_gemm_mbs(da[0], da[1], da[2], db[0], db[1], db[2], "f32", out=big[1:M + 1, 1:N + 1])
        assert torch.equal(big[1:M + 1, 1:N + 1], c32)
        big[1:M + 1, 1:N + 1] = -3.0
        assert bool((big == -3.0).all())


# ------------------------------------------------------------------------------------------------
# The other workload configurations at their real shapes
# ------------------------------------------------------------------------------------------------
def test_config_decode_skinny(mx, oracle):
    """M = 16 activations quantized online against offline-quantized weights, N = 4096 and 14336: the whole
    output against the oracle."""
    from paper_2603_08713_amd import synth

    for n in (4096, 14336):
        a_bits, w_bits = synth.decode_skinny(n, 4096)
        a = mx.mx_quantize_mbs(dev_bf16(a_bits), "oas")
        b = mx.mx_quantize_mbs(dev_bf16(w_bits), "oas")
        ah, bh = [host(t) for t in a], [host(t) for t in b]
        assert all(np.array_equal(x, y) for x, y in zip(ah, oracle.quantize(a_bits, "oas", mbs=True)))
        c = mx.mx_gemm_mbs(a[0], a[1], a[2], b[0], b[1], b[2], "f32")
        assert_gemm_close(host(c), oracle.gemm(ah, bh), "decode skinny N=%d" % n)
        assert torch.equal(mx.mx_gemm_mbs(a[0], a[1], a[2], b[0], b[1], b[2], "bf16"), c.to(torch.bfloat16))


_LLAMA70B = {}


def llama70b_operands(mx):
    """The Llama-3-70B FFN tensors, quantized on the GPU (shared by the two tests below: drawing them takes seconds)."""
    if not _LLAMA70B:
        from paper_2603_08713_amd import synth

        a_bits, w_bits = synth.llama70b_ffn(8192, 28672, 8192)
        _LLAMA70B.update(a_bits=a_bits, w_bits=w_bits, a=mx.mx_quantize_mbs(dev_bf16(a_bits), "oas"),
                         b=mx.mx_quantize_mbs(dev_bf16(w_bits), "oas"))
    return _LLAMA70B


def test_config_llama70b_ffn_sampled(mx, oracle):
    """M = 8192, N = 28672, K = 8192, the benchmark's shape and launch: quantized operands bit-exact on sampled
    rows; the MBS GEMM against the oracle on one output row of every 32-row fragment (256 rows, all columns)."""
    M, N = 8192, 28672
    d = llama70b_operands(mx)
    a, b = d["a"], d["b"]
    rows = fragment_rows(M, 70)
    wrows = np.sort(np.random.default_rng(70).choice(N, 64, replace=False))
    ah = [host(t[torch.from_numpy(rows).cuda()]) for t in a]
    assert all(np.array_equal(x, y) for x, y in zip(ah, oracle.quantize(d["a_bits"][rows], "oas", mbs=True)))
    bw = [host(t[torch.from_numpy(wrows).cuda()]) for t in b]
    assert all(np.array_equal(x, y) for x, y in zip(bw, oracle.quantize(d["w_bits"][wrows], "oas", mbs=True)))
    bh = [host(t) for t in b]
    c = mx.mx_gemm_mbs(a[0], a[1], a[2], b[0], b[1], b[2], "bf16")
    c32 = mx.mx_gemm_mbs(a[0], a[1], a[2], b[0], b[1], b[2], "f32")
    assert torch.equal(c, c32.to(torch.bfloat16))
    assert bool(torch.isfinite(c32).all())
    assert_gemm_close(host(c32[torch.from_numpy(rows).cuda()]), oracle.gemm(ah, bh), "llama70b mbs, a row of every fragment")


def test_config_llama70b_ffn_plain_sampled(mx, oracle):
    """The same shape without MBS words (256 x 256 tiles): two rows of every 256-row tile-row, in different
    fragments, against the oracle (64 rows, all columns)."""
    M = 8192
    d = llama70b_operands(mx)
    a, b = d["a"], d["b"]
    rows = fragment_rows(M, 71)
    rows = np.sort(np.concatenate([rows[(np.arange(32) * 8 + np.arange(32) % 8)], rows[(np.arange(32) * 8 + (np.arange(32) + 4) % 8)]]))
    ah = [host(t[torch.from_numpy(rows).cuda()]) for t in a]
    bh = [host(t) for t in b]
    p32 = mx.mx_gemm(a[0], a[1], b[0], b[1], "f32")
    assert torch.equal(mx.mx_gemm(a[0], a[1], b[0], b[1], "bf16"), p32.to(torch.bfloat16))
    want = oracle.gemm((ah[0], ah[1], None), (bh[0], bh[1], None))
    assert_gemm_close(host(p32[torch.from_numpy(rows).cuda()]), want, "llama70b plain sampled rows")
    _LLAMA70B.clear()


def test_config_llama70b_ffn_launches_agree_under_disturbance(mx):
    """The benchmark's shape again: the wavefronts of a workgroup synchronise every other stage only and may drift two
    stages apart, so the timing of a launch varies with what else the memory system is doing.  Launches alternate with
    a large fill that evicts the caches, in all three MBS forms and the plain one; every output must equal the first
    launch's bit for bit (a difference would be a synchronisation hole)."""
    t = llama70b_operands(mx)
    a, b = t["a"], t["b"]
    forms = {
        "both": lambda out: mx.mx_gemm_mbs(*a, *b, "bf16", out=out),
        "a only": lambda out: mx.mx_gemm_mbs(*a, b[0], b[1], None, "bf16", out=out),
        "b only": lambda out: mx.mx_gemm_mbs(a[0], a[1], None, *b, "bf16", out=out),
        "plain": lambda out: mx.mx_gemm(a[0], a[1], b[0], b[1], "bf16", out=out),
    }
    junk = torch.empty(384 * 1024 * 1024, dtype=torch.uint8, device="cuda")
    first = torch.empty((8192, 28672), dtype=torch.bfloat16, device="cuda")
    again = torch.empty_like(first)
    for name, run in forms.items():
        run(first)
        for rep in range(6):
            if rep % 2 == 0:
                junk.fill_(rep)
            again.fill_(0)
            run(again)
            assert torch.equal(first, again), (name, rep)
    del junk, first, again


def test_config_moe_grouped_sampled(mx, oracle):
    """32 experts of 2880 x 2880, 8192 tokens routed top-4 with Zipf load (32768 rows in expert order): rows
    sampled from every non-empty expert against the oracle; K = 2880 ends in a half macro block."""
    from paper_2603_08713_amd import synth

    x_bits, w_bits, offsets, token_of_row = synth.moe()
    G, dim = 32, 2880
    xa = dev_bf16(x_bits[token_of_row])               # activations gathered into expert order
    a = mx.mx_quantize_mbs(xa, "oas")
    b = mx.mx_quantize_mbs(dev_bf16(w_bits), "oas")
    off = torch.from_numpy(np.asarray(offsets, dtype=np.int64)).cuda()
    c = mx.mx_gemm_mbs_grouped(a[0], a[1], a[2], b[0], b[1], b[2], off, dim, "f32")
    torch.cuda.synchronize()
    assert bool(torch.isfinite(c).all())
    rng = np.random.default_rng(5)
    ah, bh = [host(t) for t in a], [host(t) for t in b]
    for e in range(G):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if lo == hi:
            continue
        rows = np.unique(np.concatenate([[lo, hi - 1], rng.integers(lo, hi, 2)]))
        want = oracle.gemm(tuple(t[rows] for t in ah), tuple(t[e * dim:(e + 1) * dim] for t in bh))
        assert_gemm_close(host(c[torch.from_numpy(rows).cuda()]), want, "moe expert %d" % e)
    sample = np.sort(rng.choice(len(token_of_row), 64, replace=False))
    want_q = oracle.quantize(x_bits[token_of_row[sample]], "oas", mbs=True)
    assert all(np.array_equal(t[sample], y) for t, y in zip(ah, want_q))
