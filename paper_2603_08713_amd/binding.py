"""ctypes binding of ``libmx4.so`` (C ABI in ``include/mx4.h``), same names as the C entry points.

Marshalling only: tensors in, ``data_ptr()`` + sizes + the current HIP stream out.  Output tensors
are allocated with torch when the caller does not pass them.  Nothing is computed here.
"""
from __future__ import annotations

import contextlib
import ctypes
import os
import threading
from typing import Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmx4.so")

MX_RULE_OCP, MX_RULE_FLOOR, MX_RULE_OAS = 0, 1, 2
MX_OUT_F32, MX_OUT_BF16 = 0, 1
MX_ELEM_E2M1, MX_ELEM_E4M3, MX_ELEM_E5M2, MX_ELEM_E2M3, MX_ELEM_E3M2 = 0, 1, 2, 3, 4
_ELEMS = {"e2m1": MX_ELEM_E2M1, "e4m3": MX_ELEM_E4M3, "e5m2": MX_ELEM_E5M2, "e2m3": MX_ELEM_E2M3, "e3m2": MX_ELEM_E3M2}
_RULES = {"ocp": MX_RULE_OCP, "floor": MX_RULE_FLOOR, "oas": MX_RULE_OAS}

_lib: Optional[ctypes.CDLL] = None


class MxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, mx_status_string(status), status))


def load_library() -> ctypes.CDLL:
    """Load the in-tree HIP library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libmx4.so is missing: build it with `python -m paper_2603_08713_amd.build` "
            "(or __graft_entry__.build()); this package has no CPU fallback")
    L = ctypes.CDLL(_LIB_PATH)
    i64, i32, vp, ci = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int
    L.mx_quantize.restype = ci
    L.mx_quantize.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp]
    L.mx_quantize_oas.restype = ci
    L.mx_quantize_oas.argtypes = [vp, i64, i64, i64, vp, vp, vp]
    L.mx_quantize_mbs.restype = ci
    L.mx_quantize_mbs.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp, vp]
    L.mx_quantize_mbs_pair.restype = ci
    L.mx_quantize_mbs_pair.argtypes = [vp, i64, i64, vp, vp, vp, vp, i64, i64, vp, vp, vp, i64, ci, vp]
    L.mx_gemm_mbs_quantize_a.restype = ci
    L.mx_gemm_mbs_quantize_a.argtypes = [vp, i64, ci, ci, vp, vp, vp, i64, i64, i64, ci, vp, i64, vp]
    L.mx_quantize_mbs_dynamic.restype = ci
    L.mx_quantize_mbs_dynamic.argtypes = [vp, i64, i64, i64, ci, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          vp, vp, vp, vp]
    L.mx_mbs_lut_build.restype = ci
    L.mx_mbs_lut_build.argtypes = [vp, vp]
    L.mx_quantize_mbs_dynamic_lut.restype = ci
    L.mx_quantize_mbs_dynamic_lut.argtypes = [vp, i64, i64, i64, ci, vp, ci, vp, vp, vp, vp]
    L.mx_quantize_mbs_dynamic_lut_static.restype = ci
    L.mx_quantize_mbs_dynamic_lut_static.argtypes = [vp, i64, i64, i64, ci, ci, vp, vp, vp, vp]
    L.mx_dequantize.restype = ci
    L.mx_dequantize.argtypes = [vp, vp, vp, i64, i64, ci, vp, i64, vp]
    L.mx_gemm.restype = ci
    L.mx_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp, i64, vp]
    L.mx_gemm_mbs.restype = ci
    L.mx_gemm_mbs.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, vp, i64, vp]
    L.mx_gemm_mbs_grouped.restype = ci
    L.mx_gemm_mbs_grouped.argtypes = [vp, vp, vp, vp, vp, vp, i32, vp, i64, i64, i64, ci, vp, i64, vp]
    L.mx_quantize_elem.restype = ci
    L.mx_quantize_elem.argtypes = [ci, vp, i64, i64, i64, ci, ci, vp, vp, vp, vp]
    L.mx_dequantize_elem.restype = ci
    L.mx_dequantize_elem.argtypes = [ci, vp, vp, vp, i64, i64, ci, vp, i64, vp]
    L.mx_gemm_mbs_elem.restype = ci
    L.mx_gemm_mbs_elem.argtypes = [ci, vp, vp, vp, ci, vp, vp, vp, i64, i64, i64, ci, vp, i64, vp]
    L.mx_status_string.restype = ctypes.c_char_p
    L.mx_status_string.argtypes = [ci]
    L.mx_version.restype = ci
    L.mx_version.argtypes = []
    L.mx_internal_quantize.restype = ci
    L.mx_internal_quantize.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, vp, vp, vp]
    L.mx_internal_quantize_elem.restype = ci
    L.mx_internal_quantize_elem.argtypes = [ci, vp, i64, i64, i64, ci, ci, ci, vp, vp, vp, vp]
    L.mx_internal_gemm.restype = ci
    L.mx_internal_gemm.argtypes = [vp, vp, vp, vp, vp, vp, ci, i32, vp, i64, i64, i64, ci, vp, i64, ci, ci, vp]
    L.mx_internal_gemm_plan.restype = ci
    L.mx_internal_gemm_plan.argtypes = [i64, i64, i64, ci, ci, ci, ctypes.c_char_p, ci]
    L.mx_quantize_elem_mbs_dynamic.restype = ci
    L.mx_quantize_elem_mbs_dynamic.argtypes = [ci, vp, i64, i64, i64, ci, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                               vp, vp, vp, vp]
    L.mx_gemm_mbs_elem_grouped.restype = ci
    L.mx_gemm_mbs_elem_grouped.argtypes = [ci, vp, vp, vp, ci, vp, vp, vp, ctypes.c_int32, vp, i64, i64, i64, ci, vp, i64, vp]
    L.mx_internal_gemm_elem.restype = ci
    L.mx_internal_gemm_elem.argtypes = [ci, vp, vp, vp, ci, vp, vp, vp, i64, i64, i64, ci, vp, i64, ci, vp]
    _lib = L
    return L


def mx_status_string(status: int) -> str:
    return load_library().mx_status_string(int(status)).decode()


def mx_version() -> int:
    return load_library().mx_version()


# ---- development routing (tests only) ----------------------------------------------------------------
# The library keeps no switches.  Its development entry points (csrc/mx_internal.h) take the choice of
# implementation as one more argument of the call; `forced(...)` makes the functions below pass such a
# choice, for the calling thread, while the block runs.
_dev = threading.local()


@contextlib.contextmanager
def forced(**choices):
    """quantize_hw / quantize_elem_hw = 0 or 1 (rounding implementation), gemm_shape = a kernel form and
    tile shape code of mx_gemm.hip, gemm_elem = which kernel takes an 8-/6-bit GEMM (1 = the main kernel's general
    form, 2 = the main kernel in the form the problem allows, 3 = the few-row kernel)."""
    allowed = {"quantize_hw", "quantize_elem_hw", "gemm_shape", "gemm_elem"}
    if set(choices) - allowed:
        raise TypeError("unknown choice: %s" % sorted(set(choices) - allowed))
    old = getattr(_dev, "choices", {})
    _dev.choices = dict(old, **choices)
    try:
        yield
    finally:
        _dev.choices = old


def _forced(name):
    return getattr(_dev, "choices", {}).get(name)


def gemm_plan(M: int, N: int, K: int, a_has_mbs: bool = True, b_has_mbs: bool = True, grouped: bool = False) -> str:
    """The kernel the dispatcher of mx_gemm / mx_gemm_mbs / mx_gemm_mbs_grouped picks for a problem with aligned
    arrays (host only; reported by the benchmark beside its timings)."""
    buf = ctypes.create_string_buffer(512)
    _check(load_library().mx_internal_gemm_plan(M, N, K, int(a_has_mbs), int(b_has_mbs), int(grouped), buf, 512),
           "mx_internal_gemm_plan")
    return buf.value.decode()


def _quantize_call(where, x, rows, K, ldx, rule, use_mbs, codes, scales, mbs, public):
    hw = _forced("quantize_hw")
    if hw is None:
        _check(public(), where)
    else:
        _check(load_library().mx_internal_quantize(_ptr(x), rows, K, ldx, rule, int(use_mbs), int(hw), _ptr(codes),
                                                   _ptr(scales), _ptr(mbs), _stream()), where + " (mx_internal_quantize)")


def _gemm_call(where, a, b, grouped, num_groups, row_offsets, M, N, K, code, out, ldc, mbs_entry, public):
    shape = _forced("gemm_shape")
    if shape is None:
        _check(public(), where)
    else:
        _check(load_library().mx_internal_gemm(_ptr(a[0]), _ptr(a[1]), _ptr(a[2]), _ptr(b[0]), _ptr(b[1]), _ptr(b[2]),
                                               int(grouped), int(num_groups), _ptr(row_offsets), M, N, K, code, _ptr(out),
                                               ldc, int(mbs_entry), int(shape), _stream()), where + " (mx_internal_gemm)")


# ---- helpers ---------------------------------------------------------------------------------------
def _torch():
    import torch

    return torch


def _rule(rule) -> int:
    return _RULES[rule] if isinstance(rule, str) else int(rule)


def _elem(elem) -> int:
    return _ELEMS[elem] if isinstance(elem, str) else int(elem)


def _stream() -> int:
    return _torch().cuda.current_stream().cuda_stream


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _check(status: int, where: str):
    if status != 0:
        raise MxError(status, where)


def _rows_ld(x):
    torch = _torch()
    if x.dim() != 2 or x.dtype != torch.bfloat16 or not x.is_cuda:
        raise TypeError("expected a 2-D bf16 CUDA tensor")
    if x.shape[1] > 1 and x.stride(1) != 1:
        raise ValueError("innermost dimension must be contiguous")
    return x.shape[0], x.shape[1], (x.stride(0) if x.shape[0] > 1 else max(x.stride(0), x.shape[1]))


def _u8(t, shape, name):
    torch = _torch()
    if t.dtype != torch.uint8 or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != tuple(shape):
        raise TypeError("%s must be a contiguous uint8 CUDA tensor of shape %s" % (name, tuple(shape)))
    return t


def _alloc_outputs(x, rows, K, codes, scales, mbs, want_mbs):
    torch = _torch()
    if codes is None:
        codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device)
    if want_mbs and mbs is None:
        mbs = torch.empty((rows, (K + 127) // 128), dtype=torch.uint8, device=x.device)
    _u8(codes, (rows, K // 2), "codes")
    _u8(scales, (rows, K // 32), "scales")
    if want_mbs:
        _u8(mbs, (rows, (K + 127) // 128), "mbs")
    return codes, scales, mbs


# ---- entry points ----------------------------------------------------------------------------------
def mx_quantize(x, rule="ocp", codes=None, scales=None):
    """bf16 [rows, K] -> (codes uint8 [rows, K/2], scales uint8 [rows, K/32]) with `rule`, no MBS."""
    rows, K, ldx = _rows_ld(x)
    codes, scales, _ = _alloc_outputs(x, rows, K, codes, scales, None, False)
    _quantize_call("mx_quantize", x, rows, K, ldx, _rule(rule), False, codes, scales, None,
                   lambda: load_library().mx_quantize(_ptr(x), rows, K, ldx, _rule(rule), _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


def mx_quantize_oas(x, codes=None, scales=None):
    rows, K, ldx = _rows_ld(x)
    codes, scales, _ = _alloc_outputs(x, rows, K, codes, scales, None, False)
    _quantize_call("mx_quantize_oas", x, rows, K, ldx, MX_RULE_OAS, False, codes, scales, None,
                   lambda: load_library().mx_quantize_oas(_ptr(x), rows, K, ldx, _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


def mx_quantize_mbs(x, rule="oas", codes=None, scales=None, mbs=None):
    """MBS-Static quantization -> (codes, scales, mbs uint8 [rows, ceil(K/128)])."""
    rows, K, ldx = _rows_ld(x)
    codes, scales, mbs = _alloc_outputs(x, rows, K, codes, scales, mbs, True)
    _quantize_call("mx_quantize_mbs", x, rows, K, ldx, _rule(rule), True, codes, scales, mbs,
                   lambda: load_library().mx_quantize_mbs(_ptr(x), rows, K, ldx, _rule(rule), _ptr(codes), _ptr(scales),
                                                          _ptr(mbs), _stream()))
    return codes, scales, mbs


def mx_quantize_mbs_pair(x0, x1, rule="oas", out0=None, out1=None):
    """MBS-Static quantization of two tensors with the same K in one launch -> ((codes, scales, mbs), (...))."""
    rows0, K, ld0 = _rows_ld(x0)
    rows1, K1, ld1 = _rows_ld(x1)
    if K != K1:
        raise ValueError("the two tensors must share K")
    o0 = _alloc_outputs(x0, rows0, K, *(out0 or (None, None, None)), True)
    o1 = _alloc_outputs(x1, rows1, K, *(out1 or (None, None, None)), True)
    _check(load_library().mx_quantize_mbs_pair(_ptr(x0), rows0, ld0, _ptr(o0[0]), _ptr(o0[1]), _ptr(o0[2]),
                                               _ptr(x1), rows1, ld1, _ptr(o1[0]), _ptr(o1[1]), _ptr(o1[2]),
                                               K, _rule(rule), _stream()), "mx_quantize_mbs_pair")
    return o0, o1


def mx_quantize_mbs_dynamic(x, rule="oas", cand_first=0, cand_count=16, cand_stride=16, codes=None, scales=None,
                            mbs=None):
    """MBS-Dynamic quantization (searched word per 1x128 window) -> (codes, scales, mbs)."""
    rows, K, ldx = _rows_ld(x)
    codes, scales, mbs = _alloc_outputs(x, rows, K, codes, scales, mbs, True)
    _check(load_library().mx_quantize_mbs_dynamic(_ptr(x), rows, K, ldx, _rule(rule), int(cand_first),
                                                  int(cand_count), int(cand_stride), _ptr(codes), _ptr(scales),
                                                  _ptr(mbs), _stream()), "mx_quantize_mbs_dynamic")
    return codes, scales, mbs


def mx_mbs_lut_build(lut=None):
    """The table of squared relative errors MBS-Dynamic reads (2 x 64 points x 16 slots, fp16 bit patterns as int16)."""
    torch = _torch()
    if lut is None:
        lut = torch.empty((2, 64, 16), dtype=torch.int16, device="cuda")
    if lut.dtype != torch.int16 or not lut.is_cuda or not lut.is_contiguous() or lut.numel() != 2048:
        raise TypeError("lut must be a contiguous int16 CUDA tensor of 2048 elements")
    _check(load_library().mx_mbs_lut_build(_ptr(lut), _stream()), "mx_mbs_lut_build")
    return lut


def mx_quantize_mbs_dynamic_lut(x, lut, rule="oas", keep_static=True, codes=None, scales=None, mbs=None):
    """MBS-Dynamic quantization through the table (word 16 j* of least tabulated cost per 1x128 window) -> (codes, scales, mbs)."""
    torch = _torch()
    rows, K, ldx = _rows_ld(x)
    if lut.dtype != torch.int16 or not lut.is_cuda or not lut.is_contiguous() or lut.numel() != 2048:
        raise TypeError("lut must be a contiguous int16 CUDA tensor of 2048 elements")
    codes, scales, mbs = _alloc_outputs(x, rows, K, codes, scales, mbs, True)
    _check(load_library().mx_quantize_mbs_dynamic_lut(_ptr(x), rows, K, ldx, _rule(rule), _ptr(lut), int(bool(keep_static)),
                                                      _ptr(codes), _ptr(scales), _ptr(mbs), _stream()),
           "mx_quantize_mbs_dynamic_lut")
    return codes, scales, mbs


def mx_quantize_mbs_dynamic_lut_static(x, codes, scales, mbs, rule="oas", keep_static=True):
    """mx_quantize_mbs_dynamic_lut on the table the library keeps per GPU; the call allocates nothing, so the
    caller passes the three output tensors ([rows, K/2], [rows, K/32], [rows, ceil(K/128)], uint8)."""
    rows, K, ldx = _rows_ld(x)
    _alloc_outputs(x, rows, K, codes, scales, mbs, True)  # given all three, this only checks them
    _check(load_library().mx_quantize_mbs_dynamic_lut_static(_ptr(x), rows, K, ldx, _rule(rule), int(bool(keep_static)),
                                                             _ptr(codes), _ptr(scales), _ptr(mbs), _stream()),
           "mx_quantize_mbs_dynamic_lut_static")
    return codes, scales, mbs


def _out_dtype(dtype) -> Tuple[int, object]:
    torch = _torch()
    if dtype in (MX_OUT_F32, "f32", "fp32", torch.float32):
        return MX_OUT_F32, torch.float32
    if dtype in (MX_OUT_BF16, "bf16", torch.bfloat16):
        return MX_OUT_BF16, torch.bfloat16
    raise ValueError("output dtype must be fp32 or bf16")


def mx_dequantize(codes, scales, mbs=None, out_dtype="f32", out=None):
    torch = _torch()
    rows, K = codes.shape[0], codes.shape[1] * 2
    code, tdt = _out_dtype(out_dtype)
    if out is None:
        out = torch.empty((rows, K), dtype=tdt, device=codes.device)
    if out.dtype != tdt or out.dim() != 2 or tuple(out.shape) != (rows, K) or (K > 1 and out.stride(1) != 1):
        raise TypeError("out must be [rows, K] of the requested dtype with a contiguous last dimension")
    ldo = out.stride(0) if rows > 1 else max(out.stride(0), K)
    _check(load_library().mx_dequantize(_ptr(codes), _ptr(scales), _ptr(mbs), rows, K, code, _ptr(out), ldo,
                                        _stream()), "mx_dequantize")
    return out


def _c_tensor(M, N, out_dtype, out, device):
    torch = _torch()
    code, tdt = _out_dtype(out_dtype)
    if out is None:
        out = torch.empty((M, N), dtype=tdt, device=device)
    if out.dtype != tdt or tuple(out.shape) != (M, N) or (N > 1 and out.stride(1) != 1):
        raise TypeError("C must be [M, N] of the requested dtype with a contiguous last dimension")
    ldc = out.stride(0) if M > 1 else max(out.stride(0), N)
    return code, out, ldc


def mx_gemm(a_codes, a_scales, b_codes, b_scales, out_dtype="f32", out=None):
    """Plain MXFP4 GEMM: C[M,N] = A[M,K] . B[N,K]^T."""
    M, K = a_codes.shape[0], a_codes.shape[1] * 2
    N = b_codes.shape[0]
    if b_codes.shape[1] * 2 != K:
        raise ValueError("A and B disagree on K")
    code, out, ldc = _c_tensor(M, N, out_dtype, out, a_codes.device)
    _gemm_call("mx_gemm", (a_codes, a_scales, None), (b_codes, b_scales, None), False, 0, None, M, N, K, code, out, ldc, False,
               lambda: load_library().mx_gemm(_ptr(a_codes), _ptr(a_scales), _ptr(b_codes), _ptr(b_scales), M, N, K, code,
                                              _ptr(out), ldc, _stream()))
    return out


def mx_gemm_mbs(a_codes, a_scales, a_mbs, b_codes, b_scales, b_mbs, out_dtype="f32", out=None):
    """GEMM with the per-macro-block MBS correction; a_mbs / b_mbs may be None."""
    M, K = a_codes.shape[0], a_codes.shape[1] * 2
    N = b_codes.shape[0]
    if b_codes.shape[1] * 2 != K:
        raise ValueError("A and B disagree on K")
    code, out, ldc = _c_tensor(M, N, out_dtype, out, a_codes.device)
    _gemm_call("mx_gemm_mbs", (a_codes, a_scales, a_mbs), (b_codes, b_scales, b_mbs), False, 0, None, M, N, K, code, out, ldc,
               True, lambda: load_library().mx_gemm_mbs(_ptr(a_codes), _ptr(a_scales), _ptr(a_mbs), _ptr(b_codes),
                                                        _ptr(b_scales), _ptr(b_mbs), M, N, K, code, _ptr(out), ldc, _stream()))
    return out


def elem_code_bytes(elem, K: int) -> int:
    """Bytes of a row of K codes: one per element for the 8-bit formats, 6-bit codes packed for E2M3 / E3M2."""
    return K * 3 // 4 if _elem(elem) in (MX_ELEM_E2M3, MX_ELEM_E3M2) else K


def mx_quantize_elem(x, elem="e4m3", rule="oas", use_mbs=True, codes=None, scales=None, mbs=None):
    """Quantize into an 8-bit (codes one per byte) or 6-bit (packed) MX element format, with or without MBS words."""
    torch = _torch()
    rows, K, ldx = _rows_ld(x)
    if codes is None:
        codes = torch.empty((rows, elem_code_bytes(elem, K)), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=x.device)
    if use_mbs and mbs is None:
        mbs = torch.empty((rows, (K + 127) // 128), dtype=torch.uint8, device=x.device)
    _u8(codes, (rows, elem_code_bytes(elem, K)), "codes")
    _u8(scales, (rows, K // 32), "scales")
    if use_mbs:
        _u8(mbs, (rows, (K + 127) // 128), "mbs")
    hw = _forced("quantize_elem_hw")
    if hw is None:
        _check(load_library().mx_quantize_elem(_elem(elem), _ptr(x), rows, K, ldx, _rule(rule), int(bool(use_mbs)),
                                               _ptr(codes), _ptr(scales), _ptr(mbs) if use_mbs else None, _stream()),
               "mx_quantize_elem")
    else:
        _check(load_library().mx_internal_quantize_elem(_elem(elem), _ptr(x), rows, K, ldx, _rule(rule), int(bool(use_mbs)),
                                                        int(hw), _ptr(codes), _ptr(scales), _ptr(mbs) if use_mbs else None,
                                                        _stream()), "mx_quantize_elem (mx_internal_quantize_elem)")
    return codes, scales, (mbs if use_mbs else None)


def mx_quantize_elem_mbs_dynamic(x, elem, rule="oas", cand_first=0, cand_count=16, cand_stride=16, codes=None, scales=None,
                                 mbs=None):
    """MBS-Dynamic into an 8-bit or 6-bit element format: the word of every 1x128 window searched among the static
    word and cand_count candidates for the least squared error.  Returns (codes, scales, mbs)."""
    torch = _torch()
    rows, K, ldx = _rows_ld(x)
    dev = x.device
    codes = torch.empty((rows, elem_code_bytes(elem, K)), dtype=torch.uint8, device=dev) if codes is None else codes
    scales = torch.empty((rows, K // 32), dtype=torch.uint8, device=dev) if scales is None else scales
    mbs = torch.empty((rows, (K + 127) // 128), dtype=torch.uint8, device=dev) if mbs is None else mbs
    _u8(codes, (rows, elem_code_bytes(elem, K)), "codes")
    _u8(scales, (rows, K // 32), "scales")
    _u8(mbs, (rows, (K + 127) // 128), "mbs")
    _check(load_library().mx_quantize_elem_mbs_dynamic(_elem(elem), _ptr(x), rows, K, ldx, _rule(rule), int(cand_first),
                                                       int(cand_count), int(cand_stride), _ptr(codes), _ptr(scales),
                                                       _ptr(mbs), _stream()), "mx_quantize_elem_mbs_dynamic")
    return codes, scales, mbs


def mx_dequantize_elem(elem, codes, scales, mbs=None, out_dtype="f32", out=None):
    """Dequantize codes of an 8-bit (one per byte) or 6-bit (packed) MX element format to fp32 or bf16.  K is taken
    from the scale array."""
    torch = _torch()
    rows, K = codes.shape[0], scales.shape[1] * 32
    if codes.shape[1] != elem_code_bytes(elem, K):
        raise ValueError("the code array does not have the row length of its format")
    code, dt = _out_dtype(out_dtype)
    if out is None:
        out = torch.empty((rows, K), dtype=dt, device=codes.device)
    if out.dtype != dt or out.dim() != 2 or tuple(out.shape) != (rows, K) or (K > 1 and out.stride(1) != 1):
        raise TypeError("out must be [rows, K] of the requested dtype with a contiguous last dimension")
    ldo = out.stride(0) if rows > 1 else max(out.stride(0), K)
    _check(load_library().mx_dequantize_elem(_elem(elem), _ptr(codes), _ptr(scales), _ptr(mbs), rows, K, code, _ptr(out),
                                             ldo, _stream()), "mx_dequantize_elem")
    return out


def mx_gemm_mbs_elem(a_elem, a_codes, a_scales, a_mbs, b_elem, b_codes, b_scales, b_mbs, out_dtype="f32", out=None):
    """GEMM with the MBS correction for operands in 8-bit or (packed) 6-bit MX element formats; a_mbs / b_mbs may
    be None.  K is taken from the scale arrays."""
    M, N, K = a_codes.shape[0], b_codes.shape[0], a_scales.shape[1] * 32
    if b_scales.shape[1] * 32 != K or a_codes.shape[1] != elem_code_bytes(a_elem, K) or b_codes.shape[1] != elem_code_bytes(b_elem, K):
        raise ValueError("A and B disagree on K, or a code array does not have the row length of its format")
    code, out, ldc = _c_tensor(M, N, out_dtype, out, a_codes.device)
    if _forced("gemm_elem"):
        _check(load_library().mx_internal_gemm_elem(_elem(a_elem), _ptr(a_codes), _ptr(a_scales), _ptr(a_mbs), _elem(b_elem),
                                                    _ptr(b_codes), _ptr(b_scales), _ptr(b_mbs), M, N, K, code, _ptr(out),
                                                    ldc, int(_forced("gemm_elem")), _stream()),
               "mx_gemm_mbs_elem (mx_internal_gemm_elem)")
    else:
        _check(load_library().mx_gemm_mbs_elem(_elem(a_elem), _ptr(a_codes), _ptr(a_scales), _ptr(a_mbs), _elem(b_elem),
                                               _ptr(b_codes), _ptr(b_scales), _ptr(b_mbs), M, N, K, code, _ptr(out), ldc,
                                               _stream()), "mx_gemm_mbs_elem")
    return out


def mx_gemm_mbs_elem_grouped(a_elem, a_codes, a_scales, a_mbs, b_elem, b_codes, b_scales, b_mbs, row_offsets, N,
                             out_dtype="f32", out=None):
    """Grouped GEMM for operands in 8-bit or 6-bit element formats: rows row_offsets[e]..row_offsets[e+1]-1 of A
    times B_e^T, B stacked [G*N, ...]."""
    torch = _torch()
    M, K = a_codes.shape[0], a_scales.shape[1] * 32
    if row_offsets.dtype != torch.int64 or not row_offsets.is_cuda or not row_offsets.is_contiguous():
        raise TypeError("row_offsets must be a contiguous int64 CUDA tensor")
    G = row_offsets.numel() - 1
    if (b_codes.shape[0] != G * N or b_scales.shape[1] * 32 != K or a_codes.shape[1] != elem_code_bytes(a_elem, K)
            or b_codes.shape[1] != elem_code_bytes(b_elem, K)):
        raise ValueError("B must hold num_groups stacked [N, K] weights in its format's row length")
    code, out, ldc = _c_tensor(M, N, out_dtype, out, a_codes.device)
    _check(load_library().mx_gemm_mbs_elem_grouped(_elem(a_elem), _ptr(a_codes), _ptr(a_scales), _ptr(a_mbs), _elem(b_elem),
                                                   _ptr(b_codes), _ptr(b_scales), _ptr(b_mbs), G, _ptr(row_offsets), M, N, K,
                                                   code, _ptr(out), ldc, _stream()), "mx_gemm_mbs_elem_grouped")
    return out


def mx_gemm_mbs_quantize_a(a, rule, b_codes, b_scales, b_mbs, out_dtype="f32", out=None, a_use_mbs=True):
    """Few-row GEMM with the bf16 activations `a` [M, K] quantized inside the kernel (M <= 64)."""
    M, K, lda = _rows_ld(a)
    N = b_codes.shape[0]
    if b_codes.shape[1] * 2 != K:
        raise ValueError("A and B disagree on K")
    code, out, ldc = _c_tensor(M, N, out_dtype, out, a.device)
    _check(load_library().mx_gemm_mbs_quantize_a(_ptr(a), lda, _rule(rule), int(bool(a_use_mbs)), _ptr(b_codes),
                                                 _ptr(b_scales), _ptr(b_mbs), M, N, K, code, _ptr(out), ldc,
                                                 _stream()), "mx_gemm_mbs_quantize_a")
    return out


def mx_gemm_mbs_grouped(a_codes, a_scales, a_mbs, b_codes, b_scales, b_mbs, row_offsets, N, out_dtype="f32",
                        out=None):
    """Grouped GEMM: rows row_offsets[e]..row_offsets[e+1]-1 of A times B_e^T, B stacked [G*N, K]."""
    torch = _torch()
    M, K = a_codes.shape[0], a_codes.shape[1] * 2
    if row_offsets.dtype != torch.int64 or not row_offsets.is_cuda or not row_offsets.is_contiguous():
        raise TypeError("row_offsets must be a contiguous int64 CUDA tensor")
    G = row_offsets.numel() - 1
    if b_codes.shape[0] != G * N or b_codes.shape[1] * 2 != K:
        raise ValueError("B must hold num_groups stacked [N, K] weights")
    code, out, ldc = _c_tensor(M, N, out_dtype, out, a_codes.device)
    _gemm_call("mx_gemm_mbs_grouped", (a_codes, a_scales, a_mbs), (b_codes, b_scales, b_mbs), True, G, row_offsets, M, N, K,
               code, out, ldc, True,
               lambda: load_library().mx_gemm_mbs_grouped(_ptr(a_codes), _ptr(a_scales), _ptr(a_mbs), _ptr(b_codes),
                                                          _ptr(b_scales), _ptr(b_mbs), G, _ptr(row_offsets), M, N, K, code,
                                                          _ptr(out), ldc, _stream()))
    return out
