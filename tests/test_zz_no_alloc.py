"""GPU test of the entry point that allocates nothing (mx_quantize_mbs_dynamic_lut_static): called through the C ABI
and compared byte for byte with mx_quantize_mbs_dynamic_lut on a table from mx_mbs_lut_build, on two calls in a row,
the second with a smaller input (the library's per-GPU table array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def mx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2603_08713_amd as mx_

    mx_.load_library()
    return mx_


def _dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def _call_static(lib, x, rule, keep_static, codes, scales, mbs):
    """The C ABI as a C caller sees it: plain pointers and sizes, the current stream, every buffer the caller's."""
    rows, K = x.shape
    vp = ctypes.c_void_p
    st = lib.mx_quantize_mbs_dynamic_lut_static(vp(x.data_ptr()), rows, K, x.stride(0), rule, keep_static,
                                                vp(codes.data_ptr()), vp(scales.data_ptr()), vp(mbs.data_ptr()),
                                                vp(torch.cuda.current_stream().cuda_stream))
    assert st == 0, "mx_quantize_mbs_dynamic_lut_static -> %d" % st


@pytest.mark.parametrize("keep_static", [1, 0])
def test_static_table_entry_point_matches_the_one_with_a_caller_table(mx, keep_static):
    from paper_2603_08713_amd import synth

    lib = mx.load_library()
    lut = mx.mx_mbs_lut_build()
    rule = {"ocp": 0, "floor": 1, "oas": 2}["oas"]
    assert mx.MX_RULE_OAS == rule
    # first a tensor of several workgroups with a ragged last macro block, then a smaller one
    shapes = [(96, 2880, 11), (5, 640, 12)]
    for rows, K, seed in shapes:
        bits = synth.gaussian(rows, K, 0.02, seed)
        x = _dev_bf16(bits)
        want = mx.mx_quantize_mbs_dynamic_lut(x, lut, "oas", bool(keep_static))
        # outputs allocated before the call; one guard row behind each must stay untouched
        codes = torch.full((rows + 1, K // 2), 0xA5, dtype=torch.uint8, device="cuda")
        scales = torch.full((rows + 1, K // 32), 0xA5, dtype=torch.uint8, device="cuda")
        mbs = torch.full((rows + 1, (K + 127) // 128), 0xA5, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        _call_static(lib, x, rule, keep_static, codes, scales, mbs)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for name, got, ref in (("codes", codes, want[0]), ("scales", scales, want[1]), ("mbs", mbs, want[2])):
            assert torch.equal(got[:rows], ref), "%s differ at %dx%d" % (name, rows, K)
            assert bool((got[rows] == 0xA5).all()), "%s: guard row written at %dx%d" % (name, rows, K)


def test_static_table_entry_point_in_a_captured_graph(mx):
    """Its callers include code under graph capture: the first call on the device is made before the capture (it looks
    the table's address up); the captured call is replayed over changing inputs, with eager work between the replays,
    and every replay equals the entry point with a caller's table."""
    from paper_2603_08713_amd import synth

    lib = mx.load_library()
    lut = mx.mx_mbs_lut_build()
    rows, K = 40, 1536
    x = _dev_bf16(synth.gaussian(rows, K, 0.02, 21))
    codes = torch.zeros((rows, K // 2), dtype=torch.uint8, device="cuda")
    scales = torch.zeros((rows, K // 32), dtype=torch.uint8, device="cuda")
    mbs = torch.zeros((rows, K // 128), dtype=torch.uint8, device="cuda")
    _call_static(lib, x, 2, 1, codes, scales, mbs)  # outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _call_static(lib, x, 2, 1, codes, scales, mbs)
    for replay in range(4):
        x.copy_(_dev_bf16(synth.gaussian(rows, K, 0.02 * (replay + 1), 30 + replay)))
        for t in (codes, scales, mbs):
            t.fill_(0xA5)                                # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = mx.mx_quantize_mbs_dynamic_lut(x, lut, "oas", True)
        assert torch.equal(codes, want[0]) and torch.equal(scales, want[1]) and torch.equal(mbs, want[2]), replay


def test_static_table_entry_point_rejects_what_the_other_rejects(mx):
    lib = mx.load_library()
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    vp = ctypes.c_void_p
    p, o = vp(x.data_ptr()), vp(out.data_ptr())
    f = lib.mx_quantize_mbs_dynamic_lut_static
    assert f(p, 4, 48, 48, 2, 1, o, o, o, None) == -1      # K % 32
    assert f(p, 4, 64, 64, 2, 1, o, o, None, None) == -2   # MBS words required
    assert f(p, 4, 64, 64, 7, 1, o, o, o, None) == -1      # no such rule
    assert f(p, 0, 64, 64, 2, 1, o, o, o, None) == 0       # nothing to do
    torch.cuda.synchronize()
