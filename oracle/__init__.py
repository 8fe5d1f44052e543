"""CPU oracle for MXFP4 + OAS + MBS (test infrastructure, NOT part of the product path).

Thin ctypes/numpy marshalling around ``mx_oracle.c``; every number is computed in that C file.
Only tests, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may import this
package; the HIP library and its Python binding never do.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mx_oracle.c")
_LIB = os.path.join(_HERE, "libmx_oracle.so")

RULE_OCP, RULE_FLOOR, RULE_OAS = 0, 1, 2
RULES = {"ocp": RULE_OCP, "floor": RULE_FLOOR, "oas": RULE_OAS}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over rows only). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, vp, ci, dbl = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        L.mxo_bf16_value.restype = dbl
        L.mxo_bf16_value.argtypes = [ctypes.c_uint16]
        L.mxo_e2m1_decode.restype = dbl
        L.mxo_e2m1_decode.argtypes = [ci]
        L.mxo_e2m1_nearest.restype = ci
        L.mxo_e2m1_nearest.argtypes = [dbl]
        L.mxo_mbs_static_m8.restype = ci
        L.mxo_mbs_static_m8.argtypes = [dbl]
        L.mxo_scale_exponent.restype = ci
        L.mxo_scale_exponent.argtypes = [dbl, ci]
        L.mxo_e8m0_from_exponent.restype = ci
        L.mxo_e8m0_from_exponent.argtypes = [ci]
        L.mxo_quantize.restype = ci
        L.mxo_quantize.argtypes = [vp, i64, i64, i64, ci, ci, ci, ci, vp, vp, vp]
        L.mxo_quantize_given_mbs.restype = ci
        L.mxo_quantize_given_mbs.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, vp, vp]
        L.mxo_mbs_sse.restype = dbl
        L.mxo_mbs_sse.argtypes = [vp, ci, ci, ci, ci]
        L.mxo_mbs_sse_rows.restype = ci
        L.mxo_mbs_sse_rows.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, vp]
        L.mxo_quantize_mbs_dynamic.restype = ci
        L.mxo_quantize_mbs_dynamic.argtypes = [vp, i64, i64, i64, ci, ci, ci, ci, ci, ci, vp, vp, vp]
        L.mxo_mbs_lut_entry.restype = dbl
        L.mxo_mbs_lut_entry.argtypes = [ci, ci, ci]
        L.mxo_mbs_lut_cost.restype = dbl
        L.mxo_mbs_lut_cost.argtypes = [vp, ci, ci, ci, ci, vp]
        L.mxo_quantize_mbs_dynamic_lut.restype = ci
        L.mxo_quantize_mbs_dynamic_lut.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, ci, vp, vp, vp]
        L.mxo_dequantize.restype = ci
        L.mxo_dequantize.argtypes = [vp, vp, vp, i64, i64, ci, ci, vp]
        L.mxo_gemm_rows.restype = ci
        L.mxo_gemm_rows.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, vp, i64, vp]
        L.mxo_matmul_bf16_rows.restype = ci
        L.mxo_matmul_bf16_rows.argtypes = [vp, i64, vp, i64, i64, i64, i64, vp, i64, vp]
        L.mxo_qsnr_db.restype = dbl
        L.mxo_qsnr_db.argtypes = [vp, vp, i64]
        L.mxo_num_threads.restype = ci
        L.mxo_set_num_threads.restype = ci
        L.mxo_set_num_threads.argtypes = [ci]
        L.mxo_elem_bits.restype = ci
        L.mxo_elem_bits.argtypes = [ci]
        L.mxo_elem_decode.restype = dbl
        L.mxo_elem_decode.argtypes = [ci, ci]
        L.mxo_elem_max.restype = dbl
        L.mxo_elem_max.argtypes = [ci]
        L.mxo_elem_nearest.restype = ci
        L.mxo_elem_nearest.argtypes = [ci, dbl]
        L.mxo_elem_scale_exponent.restype = ci
        L.mxo_elem_scale_exponent.argtypes = [ci, dbl, ci]
        L.mxo_elem_mbs_static_m8.restype = ci
        L.mxo_elem_mbs_static_m8.argtypes = [ci, dbl]
        L.mxo_elem_quantize.restype = ci
        L.mxo_elem_quantize.argtypes = [ci, vp, i64, i64, i64, ci, ci, ci, ci, vp, vp, vp]
        L.mxo_elem_quantize_given_mbs.restype = ci
        L.mxo_elem_quantize_given_mbs.argtypes = [ci, vp, i64, i64, i64, ci, ci, ci, vp, vp, vp]
        L.mxo_elem_mbs_sse_rows.restype = ci
        L.mxo_elem_mbs_sse_rows.argtypes = [ci, vp, i64, i64, i64, ci, ci, ci, vp, vp]
        L.mxo_elem_quantize_mbs_dynamic.restype = ci
        L.mxo_elem_quantize_mbs_dynamic.argtypes = [ci, vp, i64, i64, i64, ci, ci, ci, ci, ci, ci, vp, vp, vp]
        L.mxo_elem_dequantize.restype = ci
        L.mxo_elem_dequantize.argtypes = [ci, vp, vp, vp, i64, i64, ci, ci, vp]
        L.mxo_elem_gemm_rows.restype = ci
        L.mxo_elem_gemm_rows.argtypes = [ci, vp, vp, vp, ci, vp, vp, vp, i64, i64, i64, ci, ci, vp, i64, vp]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _rule(rule) -> int:
    return RULES[rule] if isinstance(rule, str) else int(rule)


# ---- scalar helpers (used by the pin tests) ---------------------------------------------------
def bf16_value(h: int) -> float:
    return lib().mxo_bf16_value(h)


def e2m1_decode(code: int) -> float:
    return lib().mxo_e2m1_decode(code)


def e2m1_nearest(y: float) -> int:
    return lib().mxo_e2m1_nearest(float(y))


def mbs_static_m8(alpha: float) -> int:
    return lib().mxo_mbs_static_m8(float(alpha))


def scale_exponent(alpha: float, rule) -> int:
    return lib().mxo_scale_exponent(float(alpha), _rule(rule))


def e8m0_from_exponent(s: int) -> int:
    return lib().mxo_e8m0_from_exponent(int(s))


def num_threads() -> int:
    return lib().mxo_num_threads()


def set_num_threads(n: int) -> int:
    """Threads of the row loops from now on; returns the previous number."""
    return lib().mxo_set_num_threads(int(n))


# ---- tensor functions --------------------------------------------------------------------------
def quantize(x_bf16: np.ndarray, rule="oas", mbs: bool = False, block: int = 32, macro: int = 128):
    """x_bf16: uint16 [rows, K] bf16 bit patterns. Returns (codes, scales, mbs_words or None)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    assert x.ndim == 2
    rows, K = x.shape
    codes = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, K // block), np.uint8)
    words = np.zeros((rows, (K + macro - 1) // macro), np.uint8) if mbs else None
    rc = lib().mxo_quantize(_ptr(x), rows, K, K, _rule(rule), int(bool(mbs)), block, macro,
                            _ptr(codes), _ptr(scales), _ptr(words))
    if rc != 0:
        raise ValueError("mxo_quantize: bad arguments")
    return codes, scales, words


def quantize_given_mbs(x_bf16: np.ndarray, words: np.ndarray, rule="oas", block: int = 32, macro: int = 128):
    """Quantize with caller-chosen MBS words [rows, ceil(K/macro)]. Returns (codes, scales, words)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    rows, K = x.shape
    words = np.ascontiguousarray(words, np.uint8)
    assert words.shape == (rows, (K + macro - 1) // macro)
    codes = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, K // block), np.uint8)
    rc = lib().mxo_quantize_given_mbs(_ptr(x), rows, K, K, _rule(rule), block, macro, _ptr(words),
                                      _ptr(codes), _ptr(scales))
    if rc != 0:
        raise ValueError("mxo_quantize_given_mbs: bad arguments")
    return codes, scales, words


# Default candidate list of MBS-Dynamic: 16 words equally spaced round the circle of factors,
# starting at the static word (the paper fixes the count, 16, but not the list).
DYNAMIC_DEFAULT = dict(cand_first=0, cand_count=16, cand_stride=16)


def quantize_mbs_dynamic(x_bf16: np.ndarray, rule="oas", cand_first: int = 0, cand_count: int = 16,
                         cand_stride: int = 16, block: int = 32, macro: int = 128):
    """MBS-Dynamic: per macro block the candidate word of least sum of squared errors. Returns (codes, scales, words)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    rows, K = x.shape
    codes = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, K // block), np.uint8)
    words = np.zeros((rows, (K + macro - 1) // macro), np.uint8)
    rc = lib().mxo_quantize_mbs_dynamic(_ptr(x), rows, K, K, _rule(rule), block, macro, cand_first,
                                        cand_count, cand_stride, _ptr(codes), _ptr(scales), _ptr(words))
    if rc != 0:
        raise ValueError("mxo_quantize_mbs_dynamic: bad arguments")
    return codes, scales, words


def mbs_sse(xm_bf16: np.ndarray, m8: int, rule="oas", block: int = 32) -> float:
    """Sum of squared errors of one macro block (1-D bf16 bit patterns) quantized with word m8 (Eq. 6 with
    the true error); -1 if the block holds a non-finite element."""
    xm = np.ascontiguousarray(xm_bf16, dtype=np.uint16)
    return float(lib().mxo_mbs_sse(_ptr(xm), xm.size, int(m8), _rule(rule), block))


def mbs_sse_rows(x_bf16: np.ndarray, words: np.ndarray, rule="oas", block: int = 32, macro: int = 128) -> np.ndarray:
    """The same sum for every macro block of x under the given words [rows, ceil(K/macro)]; fp64 [rows, nmac]."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    rows, K = x.shape
    words = np.ascontiguousarray(words, np.uint8)
    assert words.shape == (rows, (K + macro - 1) // macro)
    out = np.empty(words.shape, np.float64)
    rc = lib().mxo_mbs_sse_rows(_ptr(x), rows, K, K, _rule(rule), block, macro, _ptr(words), _ptr(out))
    if rc != 0:
        raise ValueError("mxo_mbs_sse_rows: bad arguments")
    return out


def mbs_lut_entry(table: int, p: int, j: int) -> float:
    """Definition of an entry of the table of Eq. 5 in fp64 (table 0 = sub-normal, 1 = normal; point p; slot j)."""
    return lib().mxo_mbs_lut_entry(int(table), int(p), int(j))


def mbs_lut() -> np.ndarray:
    """The 2 x 64 x 16 table of Eq. 5 as fp16 bit patterns (uint16), every entry the fp64 definition rounded to
    fp16 (nearest even, by numpy)."""
    t = np.array([[[mbs_lut_entry(tb, p, j) for j in range(16)] for p in range(64)] for tb in range(2)], np.float64)
    return t.astype(np.float16).view(np.uint16)


def mbs_lut_cost(xm_bf16: np.ndarray, j: int, lut: np.ndarray, rule="oas", block: int = 32) -> float:
    """Eq. 6's sum for candidate j (word 16 j) on one macro block (1-D bf16 bit patterns)."""
    xm = np.ascontiguousarray(xm_bf16, dtype=np.uint16)
    lut = np.ascontiguousarray(lut, np.uint16)
    assert lut.size == 2048
    return float(lib().mxo_mbs_lut_cost(_ptr(xm), xm.size, int(j), _rule(rule), block, _ptr(lut)))


def quantize_mbs_dynamic_lut(x_bf16: np.ndarray, lut: np.ndarray, rule="oas", keep_static: bool = True, block: int = 32,
                             macro: int = 128):
    """MBS-Dynamic with the table of Eq. 5: per macro block the word 16 j* of least tabulated cost (or the static
    word if its true error is not larger and keep_static). Returns (codes, scales, words)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    lut = np.ascontiguousarray(lut, np.uint16)
    assert lut.size == 2048
    rows, K = x.shape
    codes = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, K // block), np.uint8)
    words = np.zeros((rows, (K + macro - 1) // macro), np.uint8)
    rc = lib().mxo_quantize_mbs_dynamic_lut(_ptr(x), rows, K, K, _rule(rule), block, macro, _ptr(lut), int(bool(keep_static)),
                                            _ptr(codes), _ptr(scales), _ptr(words))
    if rc != 0:
        raise ValueError("mxo_quantize_mbs_dynamic_lut: bad arguments")
    return codes, scales, words


def dequantize(codes, scales, mbs=None, block: int = 32, macro: int = 128) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.uint8)
    mbs = None if mbs is None else np.ascontiguousarray(mbs, np.uint8)
    rows, K = codes.shape[0], codes.shape[1] * 2
    out = np.empty((rows, K), np.float64)
    rc = lib().mxo_dequantize(_ptr(codes), _ptr(scales), _ptr(mbs), rows, K, block, macro, _ptr(out))
    if rc != 0:
        raise ValueError("mxo_dequantize: bad arguments")
    return out


def gemm(a, b, rows=None, block: int = 32, macro: int = 128) -> np.ndarray:
    """a, b: (codes, scales, mbs-or-None) triples of A [M,K] and B [N,K]; returns A.B^T [len(rows), N] fp64."""
    ac, asc, am = [None if t is None else np.ascontiguousarray(t, np.uint8) for t in a]
    bc, bsc, bm = [None if t is None else np.ascontiguousarray(t, np.uint8) for t in b]
    M, K = ac.shape[0], ac.shape[1] * 2
    N = bc.shape[0]
    assert bc.shape[1] * 2 == K
    idx = None if rows is None else np.ascontiguousarray(rows, np.int64)
    n = M if idx is None else len(idx)
    C = np.empty((n, N), np.float64)
    rc = lib().mxo_gemm_rows(_ptr(ac), _ptr(asc), _ptr(am), _ptr(bc), _ptr(bsc), _ptr(bm),
                             M, N, K, block, macro, _ptr(idx), n, _ptr(C))
    if rc != 0:
        raise ValueError("mxo_gemm_rows: bad arguments")
    return C


def matmul_bf16(A_bf16, B_bf16, rows=None) -> np.ndarray:
    A = np.ascontiguousarray(A_bf16, np.uint16)
    B = np.ascontiguousarray(B_bf16, np.uint16)
    M, K = A.shape
    N = B.shape[0]
    idx = None if rows is None else np.ascontiguousarray(rows, np.int64)
    n = M if idx is None else len(idx)
    C = np.empty((n, N), np.float64)
    rc = lib().mxo_matmul_bf16_rows(_ptr(A), K, _ptr(B), K, M, N, K, _ptr(idx), n, _ptr(C))
    if rc != 0:
        raise ValueError("mxo_matmul_bf16_rows: bad arguments")
    return C


def qsnr_db(ref, test) -> float:
    r = np.ascontiguousarray(ref, np.float64).ravel()
    t = np.ascontiguousarray(test, np.float64).ravel()
    assert r.size == t.size
    return lib().mxo_qsnr_db(_ptr(r), _ptr(t), r.size)


def bf16_to_f64(x_bf16: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (the reference signal of Eq. 1)."""
    u = np.ascontiguousarray(x_bf16, np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


# ---- other MX element formats (codes one per byte) ----------------------------------------------
ELEMS = {"e2m1": 0, "e4m3": 1, "e5m2": 2, "e2m3": 3, "e3m2": 4}


def _elem(fmt) -> int:
    return ELEMS[fmt] if isinstance(fmt, str) else int(fmt)


def elem_bits(fmt) -> int:
    return lib().mxo_elem_bits(_elem(fmt))


def elem_decode(fmt, code: int) -> float:
    return lib().mxo_elem_decode(_elem(fmt), int(code))


def elem_max(fmt) -> float:
    return lib().mxo_elem_max(_elem(fmt))


def elem_nearest(fmt, y: float) -> int:
    return lib().mxo_elem_nearest(_elem(fmt), float(y))


def elem_scale_exponent(fmt, alpha: float, rule) -> int:
    return lib().mxo_elem_scale_exponent(_elem(fmt), float(alpha), _rule(rule))


def elem_mbs_static_m8(fmt, alpha: float) -> int:
    return lib().mxo_elem_mbs_static_m8(_elem(fmt), float(alpha))


def elem_quantize(fmt, x_bf16: np.ndarray, rule="oas", mbs: bool = False, block: int = 32, macro: int = 128):
    """Quantize into element format fmt. Returns (codes [rows, K] one per byte, scales, mbs words or None)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    rows, K = x.shape
    codes = np.zeros((rows, K), np.uint8)
    scales = np.zeros((rows, K // block), np.uint8)
    words = np.zeros((rows, (K + macro - 1) // macro), np.uint8) if mbs else None
    rc = lib().mxo_elem_quantize(_elem(fmt), _ptr(x), rows, K, K, _rule(rule), int(bool(mbs)), block, macro,
                                 _ptr(codes), _ptr(scales), _ptr(words))
    if rc != 0:
        raise ValueError("mxo_elem_quantize: bad arguments")
    return codes, scales, words


def elem_quantize_given_mbs(fmt, x_bf16: np.ndarray, words: np.ndarray, rule="oas", block: int = 32, macro: int = 128):
    """Quantize into element format fmt with caller-chosen MBS words. Returns (codes one per byte, scales, words)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    rows, K = x.shape
    words = np.ascontiguousarray(words, np.uint8)
    assert words.shape == (rows, (K + macro - 1) // macro)
    codes = np.zeros((rows, K), np.uint8)
    scales = np.zeros((rows, K // block), np.uint8)
    rc = lib().mxo_elem_quantize_given_mbs(_elem(fmt), _ptr(x), rows, K, K, _rule(rule), block, macro, _ptr(words),
                                           _ptr(codes), _ptr(scales))
    if rc != 0:
        raise ValueError("mxo_elem_quantize_given_mbs: bad arguments")
    return codes, scales, words


def elem_mbs_sse_rows(fmt, x_bf16: np.ndarray, words: np.ndarray, rule="oas", block: int = 32, macro: int = 128) -> np.ndarray:
    """Exact sum of squared errors (fp64) of every macro block of x in element format fmt under the given words
    [rows, ceil(K/macro)]; -1 where a macro block holds a non-finite element (Eq. 6 with the true error)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    rows, K = x.shape
    words = np.ascontiguousarray(words, np.uint8)
    assert words.shape == (rows, (K + macro - 1) // macro)
    out = np.empty(words.shape, np.float64)
    rc = lib().mxo_elem_mbs_sse_rows(_elem(fmt), _ptr(x), rows, K, K, _rule(rule), block, macro, _ptr(words), _ptr(out))
    if rc != 0:
        raise ValueError("mxo_elem_mbs_sse_rows: bad arguments")
    return out


def elem_quantize_mbs_dynamic(fmt, x_bf16: np.ndarray, rule="oas", cand_first: int = 0, cand_count: int = 16,
                              cand_stride: int = 16, block: int = 32, macro: int = 128):
    """MBS-Dynamic into element format fmt (Sec. 4.3.3 with the true error). Returns (codes, scales, words)."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16)
    rows, K = x.shape
    codes = np.zeros((rows, K), np.uint8)
    scales = np.zeros((rows, K // block), np.uint8)
    words = np.zeros((rows, (K + macro - 1) // macro), np.uint8)
    rc = lib().mxo_elem_quantize_mbs_dynamic(_elem(fmt), _ptr(x), rows, K, K, _rule(rule), block, macro, cand_first,
                                             cand_count, cand_stride, _ptr(codes), _ptr(scales), _ptr(words))
    if rc != 0:
        raise ValueError("mxo_elem_quantize_mbs_dynamic: bad arguments")
    return codes, scales, words


def elem_dequantize(fmt, codes, scales, mbs=None, block: int = 32, macro: int = 128) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.uint8)
    mbs = None if mbs is None else np.ascontiguousarray(mbs, np.uint8)
    rows, K = codes.shape
    out = np.empty((rows, K), np.float64)
    rc = lib().mxo_elem_dequantize(_elem(fmt), _ptr(codes), _ptr(scales), _ptr(mbs), rows, K, block, macro, _ptr(out))
    if rc != 0:
        raise ValueError("mxo_elem_dequantize: bad arguments")
    return out


def elem_gemm(fmt_a, a, fmt_b, b, rows=None, block: int = 32, macro: int = 128) -> np.ndarray:
    """a, b: (codes one per byte, scales, mbs-or-None) of A [M,K] and B [N,K]; A.B^T [len(rows), N] fp64."""
    ac, asc, am = [None if t is None else np.ascontiguousarray(t, np.uint8) for t in a]
    bc, bsc, bm = [None if t is None else np.ascontiguousarray(t, np.uint8) for t in b]
    M, K = ac.shape
    N = bc.shape[0]
    assert bc.shape[1] == K
    idx = None if rows is None else np.ascontiguousarray(rows, np.int64)
    n = M if idx is None else len(idx)
    C = np.empty((n, N), np.float64)
    rc = lib().mxo_elem_gemm_rows(_elem(fmt_a), _ptr(ac), _ptr(asc), _ptr(am), _elem(fmt_b), _ptr(bc), _ptr(bsc),
                                  _ptr(bm), M, N, K, block, macro, _ptr(idx), n, _ptr(C))
    if rc != 0:
        raise ValueError("mxo_elem_gemm_rows: bad arguments")
    return C


def mbs_overhead_model(tm: int = 128, tn: int = 128, tk: int = 128):
    """Analytic per-tile cost of the MBS correction (App. B, Eq. 7-8).

    Returns (extra fp32 ops / FP4 multiply ops, extra bytes / output-tile bytes): the correction is
    two fp32 operations per output element per tile (Eq. 7 counts them against the tm*tn*tk FP4
    multiplies), and it loads one 2-byte sigma per row of A and per row of B against a tm x tn fp32
    output tile (Eq. 8).
    """
    ops = (2 * tm * tn) / (tm * tn * tk)
    traffic = (2 * (tm + tn)) / (4 * tm * tn)
    return ops, traffic
