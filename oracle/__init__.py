"""CPU oracle for the Fier decode step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``fier_oracle.c`` (plain C, fp64; see that file's
header for what each function computes and the passages of the paper it
follows).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product
package never does, and this package never imports the product's kernels.

All arrays are numpy, host memory.  16-bit floats travel as raw ``uint16``
words plus a dtype code (0 = binary16, 1 = bfloat16).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fier_oracle.c")
_SO = os.path.join(_HERE, "libfier_oracle.so")

F16, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (IEEE arithmetic: no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        L = C.CDLL(_SO)
        vp, i32, f64 = C.c_void_p, C.c_int, C.c_double
        L.fier_oracle_to_f32.restype = C.c_float
        L.fier_oracle_to_f32.argtypes = [C.c_uint16, i32]
        L.fier_oracle_from_f32.restype = C.c_uint16
        L.fier_oracle_from_f32.argtypes = [C.c_float, i32]
        L.fier_oracle_quantize.restype = None
        L.fier_oracle_quantize.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, i32]
        L.fier_oracle_append.restype = None
        L.fier_oracle_append.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        L.fier_oracle_dequantize.restype = None
        L.fier_oracle_dequantize.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
        L.fier_oracle_score.restype = None
        L.fier_oracle_score.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, vp, i32]
        L.fier_oracle_topk.restype = None
        L.fier_oracle_topk.argtypes = [vp, i32, i32, vp, vp, i32, vp, vp]
        L.fier_oracle_page_minmax.restype = None
        L.fier_oracle_page_minmax.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp]
        L.fier_oracle_page_score.restype = None
        L.fier_oracle_page_score.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, vp, i32, vp]
        L.fier_oracle_page_mean.restype = None
        L.fier_oracle_page_mean.argtypes = [vp, i32, i32, i32, vp, vp]
        L.fier_oracle_expand_pages.restype = None
        L.fier_oracle_expand_pages.argtypes = [vp, vp, i32, i32, i32, vp, i32, vp, vp]
        L.fier_oracle_attention.restype = None
        L.fier_oracle_attention.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, f64, vp, vp, vp,
                                            i32, vp, i32]
        L.fier_oracle_max_threads.restype = i32
        L.fier_oracle_max_threads.argtypes = []
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, shape=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


def max_threads() -> int:
    return int(lib().fier_oracle_max_threads())


def to_f32(words: np.ndarray, dtype: int) -> np.ndarray:
    """Element-wise 16-bit word -> binary32 through the oracle's own converter."""
    L = lib()
    flat = np.asarray(words, dtype=np.uint16).ravel()
    out = np.array([L.fier_oracle_to_f32(int(w), dtype) for w in flat], dtype=np.float32)
    return out.reshape(np.shape(words))


def from_f32(x: np.ndarray, dtype: int) -> np.ndarray:
    L = lib()
    flat = np.asarray(x, dtype=np.float32).ravel()
    out = np.array([L.fier_oracle_from_f32(float(v), dtype) for v in flat], dtype=np.uint16)
    return out.reshape(np.shape(x))


def quantize(K: np.ndarray, L: np.ndarray, g: int, dtype: int, n_threads: int = 1):
    """K [U][Lcap][D] uint16 words, L [U] int32 -> bits [U][Lcap][D] u8, s, z [U][Lcap/g][D] u16."""
    U, Lcap, D = K.shape
    _chk(K, np.uint16)
    _chk(L, np.int32, (U,))
    assert Lcap % g == 0
    bits = np.zeros((U, Lcap, D), np.uint8)
    s = np.zeros((U, Lcap // g, D), np.uint16)
    z = np.zeros((U, Lcap // g, D), np.uint16)
    lib().fier_oracle_quantize(_p(K), U, Lcap, D, g, dtype, _p(L), _p(bits), _p(s), _p(z), n_threads)
    return bits, s, z


def append(K, V, L, k_new, v_new, bits, s, z, g: int, dtype: int):
    """In place: rows L[u] of K, V <- k_new, v_new; tail group of bits, s, z re-derived."""
    U, Lcap, D = K.shape
    for a in (K, V):
        _chk(a, np.uint16, (U, Lcap, D))
    _chk(L, np.int32, (U,))
    _chk(k_new, np.uint16, (U, D))
    _chk(v_new, np.uint16, (U, D))
    _chk(bits, np.uint8, (U, Lcap, D))
    _chk(s, np.uint16, (U, Lcap // g, D))
    _chk(z, np.uint16, (U, Lcap // g, D))
    lib().fier_oracle_append(_p(K), _p(V), U, Lcap, D, g, dtype, _p(L), _p(k_new), _p(v_new),
                             _p(bits), _p(s), _p(z))


def dequantize(bits, s, z, L, g: int, dtype: int) -> np.ndarray:
    U, Lcap, D = bits.shape
    _chk(bits, np.uint8)
    _chk(s, np.uint16, (U, Lcap // g, D))
    _chk(z, np.uint16, (U, Lcap // g, D))
    _chk(L, np.int32, (U,))
    Kt = np.zeros((U, Lcap, D), np.float64)
    lib().fier_oracle_dequantize(_p(bits), _p(s), _p(z), U, Lcap, D, g, dtype, _p(L), _p(Kt))
    return Kt


def score(bits, s, z, q, L, g: int, dtype: int, n_threads: int = 1) -> np.ndarray:
    """q [U][n_rep][D] uint16 -> scores [U][Lcap] fp64 (entries >= L[u] are 0)."""
    U, Lcap, D = bits.shape
    _chk(bits, np.uint8)
    _chk(s, np.uint16, (U, Lcap // g, D))
    _chk(z, np.uint16, (U, Lcap // g, D))
    _chk(q, np.uint16)
    assert q.ndim == 3 and q.shape[0] == U and q.shape[2] == D
    _chk(L, np.int32, (U,))
    out = np.zeros((U, Lcap), np.float64)
    lib().fier_oracle_score(_p(bits), _p(s), _p(z), _p(q), U, q.shape[1], Lcap, D, g, dtype, _p(L),
                            _p(out), n_threads)
    return out


def topk(scores, L, budget, max_budget: int):
    """scores [U][Lcap] fp64 -> idx [U][max_budget] int32 (ascending, -1 padded), count [U]."""
    U, Lcap = scores.shape
    _chk(scores, np.float64)
    _chk(L, np.int32, (U,))
    _chk(budget, np.int32, (U,))
    idx = np.full((U, max_budget), -1, np.int32)
    count = np.zeros((U,), np.int32)
    lib().fier_oracle_topk(_p(scores), U, Lcap, _p(L), _p(budget), max_budget, _p(idx), _p(count))
    return idx, count


def page_minmax(K, L, page: int, dtype: int):
    """Channel-wise min / max key vectors of every page (raw 16-bit words): [U][Lcap/page][D] each."""
    U, Lcap, D = K.shape
    _chk(K, np.uint16)
    _chk(L, np.int32, (U,))
    assert Lcap % page == 0
    kmin = np.zeros((U, Lcap // page, D), np.uint16)
    kmax = np.zeros_like(kmin)
    lib().fier_oracle_page_minmax(_p(K), U, Lcap, D, page, dtype, _p(L), _p(kmin), _p(kmax))
    return kmin, kmax


def page_score(kmin, kmax, q, L, page: int, dtype: int, mode: int) -> np.ndarray:
    """Page importance of Eq. 1-3 (mode 0: max over channels as printed; mode 1: sum over channels)."""
    U, NP, D = kmin.shape
    _chk(kmin, np.uint16)
    _chk(kmax, np.uint16, (U, NP, D))
    _chk(q, np.uint16)
    _chk(L, np.int32, (U,))
    n_rep = q.shape[1]
    assert q.shape == (U, n_rep, D)
    out = np.zeros((U, NP), np.float64)
    lib().fier_oracle_page_score(_p(kmin), _p(kmax), _p(q), U, n_rep, NP * page, D, page, dtype, _p(L), mode, _p(out))
    return out


def page_mean(scores, L, page: int) -> np.ndarray:
    """Average token score per page over the tokens present."""
    U, Lcap = scores.shape
    _chk(scores, np.float64)
    _chk(L, np.int32, (U,))
    out = np.zeros((U, Lcap // page), np.float64)
    lib().fier_oracle_page_mean(_p(scores), U, Lcap, page, _p(L), _p(out))
    return out


def expand_pages(page_idx, page_cnt, L, page: int, max_budget: int):
    """Tokens of the selected pages, ascending, clipped to the lengths: (idx [U][max_budget], cnt [U])."""
    U, max_pages = page_idx.shape
    _chk(page_idx, np.int32)
    _chk(page_cnt, np.int32, (U,))
    _chk(L, np.int32, (U,))
    idx = np.full((U, max_budget), -1, np.int32)
    cnt = np.zeros(U, np.int32)
    lib().fier_oracle_expand_pages(_p(page_idx), _p(page_cnt), U, max_pages, page, _p(L), max_budget, _p(idx), _p(cnt))
    return idx, cnt


def attention(K, V, q, L, sm_scale: float, dtype: int, idx=None, count=None, n_threads: int = 1):
    """Exact attention over rows idx[u][:count[u]] (idx None: all of [0, L[u])). out [U][n_rep][D] fp64."""
    U, Lcap, D = K.shape
    _chk(K, np.uint16)
    _chk(V, np.uint16, (U, Lcap, D))
    _chk(q, np.uint16)
    assert q.ndim == 3 and q.shape[0] == U and q.shape[2] == D
    _chk(L, np.int32, (U,))
    max_budget = 0
    if idx is not None:
        _chk(idx, np.int32)
        _chk(count, np.int32, (U,))
        assert idx.ndim == 2 and idx.shape[0] == U
        max_budget = idx.shape[1]
    out = np.zeros((U, q.shape[1], D), np.float64)
    lib().fier_oracle_attention(_p(K), _p(V), _p(q), U, q.shape[1], Lcap, D, dtype, float(sm_scale),
                                _p(L), _p(idx), _p(count), max_budget, _p(out), n_threads)
    return out
