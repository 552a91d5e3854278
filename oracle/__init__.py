"""ctypes front end of the CPU oracle (``spark_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only the tests, the smoke check and the
CPU-baseline leg of the benchmark import this package.  It shares nothing with
the HIP library and never imports it.

Arrays are numpy; bf16 tensors are ``uint16`` bit patterns.  K and V are
addressed as ``x[n * tok_stride + h * head_stride + j]`` (strides in elements)
so both token-major ``[total, Hkv, D]`` and head-major ``[Hkv, total, D]``
buffers can be passed without copying.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spark_oracle.c")
_LIB = os.path.join(_HERE, "libspark_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (``-O2``, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_max_threads.restype = ctypes.c_int
        _lib.oracle_prune.restype = ctypes.c_int
        _lib.oracle_prune_values.restype = ctypes.c_int
        _lib.oracle_prune_topp.restype = ctypes.c_int
        _lib.oracle_uniform.restype = ctypes.c_double
        _lib.oracle_mix32.restype = ctypes.c_uint32
    return _lib


def set_threads(n: int) -> None:
    lib().oracle_set_threads(ctypes.c_int(int(n)))


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _strided(x: np.ndarray, layout: str):
    """Return (flat uint16 array, tok_stride, head_stride, total, Hkv, D) for K or V."""
    assert x.dtype == np.uint16 and x.ndim == 3 and x.flags.c_contiguous
    if layout == "NHD":          # [total, Hkv, D]
        total, hkv, d = x.shape
        return x, hkv * d, d, total, hkv, d
    if layout == "HND":          # [Hkv, total, D]
        hkv, total, d = x.shape
        return x, d, total * d, total, hkv, d
    raise ValueError(layout)


def window_stat(qwin: np.ndarray, n_kv_heads: int):
    """qwin [B,Hq,W,D] bf16 bits -> (qbar f64 [B,Hq,D], a64 [B,Hkv,D], a32 [B,Hkv,D])."""
    qwin = _c(qwin, np.uint16)
    b, hq, w, d = qwin.shape
    assert hq % n_kv_heads == 0
    qbar = np.empty((b, hq, d), np.float64)
    a64 = np.empty((b, n_kv_heads, d), np.float64)
    a32 = np.empty((b, n_kv_heads, d), np.float32)
    lib().oracle_window_stat(_p(qwin), b, hq, n_kv_heads, w, d, _p(qbar), _p(a64), _p(a32))
    return qbar, a64, a32


@dataclass
class Pruned:
    """What the prefill step leaves behind for one layer (all rows = total * Hkv)."""
    mask: np.ndarray     # uint32 [total, Hkv, ceil(D/32)], bit j%32 of word j/32 = channel j kept
    kept: np.ndarray     # uint16 [total, Hkv, T], original bf16 bits, ascending channel
    mu64: np.ndarray     # float64 [total, Hkv]
    mu32: np.ndarray     # float32 [total, Hkv]  (what decode consumes)
    gap: np.ndarray      # float64 [total, Hkv]  relative margin between T-th and (T+1)-th saliency
    a32: np.ndarray      # float32 [B, Hkv, D]
    w: np.ndarray | None  # float32 [total, Hkv, D] when requested
    T: int
    D: int
    codes: np.ndarray | None = None   # int8 [total, Hkv, T]   (int8 storage variant)
    scale: np.ndarray | None = None   # float32 [total, Hkv]
    count: np.ndarray | None = None   # int32 [total, Hkv]  kept channels per row (top-p variant; else T everywhere)

    def near_ties(self, rel=1e-6) -> int:
        return int(np.count_nonzero(self.gap < rel))


def prune(k: np.ndarray, layout: str, a32: np.ndarray, cu: np.ndarray, T: int,
          want_w: bool = False) -> Pruned:
    k, ts, hs, total, hkv, d = _strided(k, layout)
    cu = _c(cu, np.int32)
    b = cu.shape[0] - 1
    assert int(cu[-1]) == total and int(cu[0]) == 0
    a32 = _c(a32, np.float32)
    assert a32.shape == (b, hkv, d)
    mw = (d + 31) // 32
    mask = np.empty((total, hkv, mw), np.uint32)
    kept = np.empty((total, hkv, T), np.uint16)
    mu64 = np.empty((total, hkv), np.float64)
    mu32 = np.empty((total, hkv), np.float32)
    gap = np.empty((total, hkv), np.float64)
    w = np.empty((total, hkv, d), np.float32) if want_w else None
    rc = lib().oracle_prune(_p(k), ctypes.c_int64(ts), ctypes.c_int64(hs), _p(a32), _p(cu),
                            b, hkv, d, int(T), _p(mask), _p(kept), _p(mu64), _p(mu32), _p(gap),
                            _p(w))
    if rc != 0:
        raise ValueError("oracle_prune: bad arguments")
    return Pruned(mask, kept, mu64, mu32, gap, a32, w, int(T), d)


def prune_topp(k: np.ndarray, layout: str, a32: np.ndarray, cu: np.ndarray, p_bp: int = 9900) -> Pruned:
    """The top-p variant: per (token, KV head) the fewest most salient channels whose saliencies reach
    p_bp / 10000 of the row total.  Returns a Pruned whose `kept` is [total, Hkv, D] (the first count[row]
    entries of a row are used) and whose `count` holds the per-row numbers; T = D is the row stride, so the
    decode functions take it as it is."""
    k, ts, hs, total, hkv, d = _strided(k, layout)
    cu = _c(cu, np.int32)
    b = cu.shape[0] - 1
    assert int(cu[-1]) == total and int(cu[0]) == 0
    a32 = _c(a32, np.float32)
    assert a32.shape == (b, hkv, d)
    mw = (d + 31) // 32
    mask = np.empty((total, hkv, mw), np.uint32)
    kept = np.empty((total, hkv, d), np.uint16)
    count = np.empty((total, hkv), np.int32)
    mu64 = np.empty((total, hkv), np.float64)
    mu32 = np.empty((total, hkv), np.float32)
    rc = lib().oracle_prune_topp(_p(k), ctypes.c_int64(ts), ctypes.c_int64(hs), _p(a32), _p(cu), b, hkv, d,
                                 int(p_bp), _p(mask), _p(kept), _p(count), _p(mu64), _p(mu32))
    if rc != 0:
        raise ValueError("oracle_prune_topp: bad arguments")
    pr = Pruned(mask, kept, mu64, mu32, np.full((total, hkv), np.inf), a32, None, d, d)
    pr.count = count
    return pr


def quant_int8(pr: Pruned) -> Pruned:
    rows = pr.kept.shape[0] * pr.kept.shape[1]
    codes = np.empty(pr.kept.shape, np.int8)
    scale = np.empty(pr.kept.shape[:2], np.float32)
    lib().oracle_quant_int8(_p(pr.kept), ctypes.c_int64(rows), pr.T, _p(codes), _p(scale))
    out = Pruned(pr.mask, pr.kept, pr.mu64, pr.mu32, pr.gap, pr.a32, pr.w, pr.T, pr.D)
    out.codes, out.scale = codes, scale
    return out


@dataclass
class PrunedValues:
    """The value cache after channel pruning (appendix on pruning value-cache channels)."""
    mask: np.ndarray     # uint32 [total, Hkv, ceil(D/32)]
    kept: np.ndarray     # uint16 [total, Hkv, Tv], original bf16 bits, ascending channel
    gap: np.ndarray      # float64 [total, Hkv]  relative margin between Tv-th and (Tv+1)-th |v|
    T: int
    D: int

    def near_ties(self, rel=1e-6) -> int:
        return int(np.count_nonzero(self.gap < rel))


def prune_values(v: np.ndarray, layout: str, Tv: int) -> PrunedValues:
    """Per (token, KV head): keep the Tv channels of largest |v| (ties: lower channel)."""
    v, ts, hs, total, hkv, d = _strided(v, layout)
    mw = (d + 31) // 32
    mask = np.empty((total, hkv, mw), np.uint32)
    kept = np.empty((total, hkv, Tv), np.uint16)
    gap = np.empty((total, hkv), np.float64)
    rc = lib().oracle_prune_values(_p(v), ctypes.c_int64(ts), ctypes.c_int64(hs), ctypes.c_int64(total),
                                   hkv, d, int(Tv), _p(mask), _p(kept), _p(gap))
    if rc != 0:
        raise ValueError("oracle_prune_values: bad arguments")
    return PrunedValues(mask, kept, gap, int(Tv), d)


def expand_values(pv: PrunedValues) -> np.ndarray:
    """Dense value rows as decode consumes them: kept entries at their channels, pruned entries 0.
    Returns uint16 [total, Hkv, D] (layout "NHD"); pass it as V to the decode functions."""
    total, hkv, _ = pv.mask.shape
    vt = np.empty((total, hkv, pv.D), np.uint16)
    lib().oracle_expand_values(_p(pv.mask), _p(pv.kept), ctypes.c_int64(total), hkv, pv.D, pv.T, _p(vt))
    return vt


def _decode(fn, q, pr: Pruned, v, layout, cu, scale, want_probs):
    q = _c(q, np.uint16)
    b, hq, d = q.shape
    v, ts, hs, total, hkv, dv = _strided(v, layout)
    assert dv == d == pr.D
    cu = _c(cu, np.int32)
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    out = np.empty((b, hq, d), np.float64)
    probs = np.zeros((hq, total), np.float64) if want_probs else None
    args = [_p(q), _p(pr.mask), _p(pr.kept), _p(pr.codes), _p(pr.scale), _p(pr.mu32), _p(pr.a32),
            _p(v), ctypes.c_int64(ts), ctypes.c_int64(hs), _p(cu), b, hq, hkv, d, pr.T,
            ctypes.c_double(scale), _p(out)]
    if fn == "literal":
        lib().oracle_decode_literal(*args, _p(probs))
    else:
        lib().oracle_decode_fused(*args)
    return (out, probs) if want_probs else out


def decode_literal(q, pr: Pruned, v, layout, cu, scale=None, want_probs=False):
    """The oracle of record: rebuild K-tilde row by row, then Eq. (4)."""
    return _decode("literal", q, pr, v, layout, cu, scale, want_probs)


def decode_fused(q, pr: Pruned, v, layout, cu, scale=None):
    """Algebraically identical form with the recovery term factored out."""
    return _decode("fused", q, pr, v, layout, cu, scale, False)


GAUSSIAN, EXPONENTIAL = 1, 2


def row_stats(k: np.ndarray, layout: str, a32: np.ndarray, cu: np.ndarray):
    """All-channel saliency statistics per (token, KV head): (mu float32, sigma float32), each [total, Hkv]."""
    k, ts, hs, total, hkv, d = _strided(k, layout)
    cu = _c(cu, np.int32)
    a32 = _c(a32, np.float32)
    mu = np.empty((total, hkv), np.float32)
    sigma = np.empty((total, hkv), np.float32)
    lib().oracle_row_stats(_p(k), ctypes.c_int64(ts), ctypes.c_int64(hs), _p(a32), _p(cu), cu.shape[0] - 1, hkv, d,
                           _p(mu), _p(sigma))
    return mu, sigma


def mix32(x: int) -> int:
    return int(lib().oracle_mix32(ctypes.c_uint32(x & 0xFFFFFFFF)))


def uniform(seed: int, n: int, h: int, c: int) -> float:
    return float(lib().oracle_uniform(ctypes.c_uint32(seed & 0xFFFFFFFF), ctypes.c_uint32((seed >> 32) & 0xFFFFFFFF),
                                      ctypes.c_uint32(n), ctypes.c_uint32(h), ctypes.c_uint32(c)))


def decode_sampled(kind: int, seed: int, q, pr: Pruned, mu_all, sigma, v, layout, cu, scale=None, want_ktilde=False):
    """Decode with the Gaussian (1) or Exponential (2) recovery function; seed is a 64-bit integer."""
    q = _c(q, np.uint16)
    b, hq, d = q.shape
    v, ts, hs, total, hkv, dv = _strided(v, layout)
    assert dv == d == pr.D
    cu = _c(cu, np.int32)
    mu_all, sigma = _c(mu_all, np.float32), _c(sigma, np.float32)
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    out = np.empty((b, hq, d), np.float64)
    kt = np.zeros((total, hkv, d), np.float64) if want_ktilde else None
    lib().oracle_decode_sampled(int(kind), ctypes.c_uint32(seed & 0xFFFFFFFF), ctypes.c_uint32((seed >> 32) & 0xFFFFFFFF),
                                _p(q), _p(pr.mask), _p(pr.kept), _p(pr.codes), _p(pr.scale), _p(mu_all), _p(sigma), _p(pr.a32), _p(v),
                                ctypes.c_int64(ts), ctypes.c_int64(hs), _p(cu), b, hq, hkv, d, pr.T,
                                ctypes.c_double(scale), _p(out), _p(kt))
    return (out, kt) if want_ktilde else out


def decode_literal_tail(q, pr: Pruned, v, layout, cu, tail_k, tail_v, tail_len, scale=None):
    """Decode over the pruned prefix followed by appended, never-pruned rows.
    tail_k, tail_v uint16 [B, cap, Hkv, D]; tail_len int32 [B]."""
    q = _c(q, np.uint16)
    b, hq, d = q.shape
    v, ts, hs, total, hkv, dv = _strided(v, layout)
    assert dv == d == pr.D
    cu = _c(cu, np.int32)
    tail_k, tail_v = _c(tail_k, np.uint16), _c(tail_v, np.uint16)
    tail_len = _c(tail_len, np.int32)
    cap = tail_k.shape[1]
    assert tail_k.shape == (b, cap, hkv, d) == tail_v.shape and tail_len.shape == (b,)
    assert np.all((tail_len >= 0) & (tail_len <= cap))
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    out = np.empty((b, hq, d), np.float64)
    lib().oracle_decode_literal_tail(_p(q), _p(pr.mask), _p(pr.kept), _p(pr.codes), _p(pr.scale), _p(pr.mu32),
                                     _p(pr.a32), _p(v), ctypes.c_int64(ts), ctypes.c_int64(hs), _p(cu),
                                     _p(tail_k), _p(tail_v), _p(tail_len), int(cap), b, hq, hkv, d, pr.T,
                                     ctypes.c_double(scale), _p(out))
    return out


def dense_attn(q, k, v, layout, cu, scale=None):
    """Eq. (4) on the unpruned cache."""
    q = _c(q, np.uint16)
    b, hq, d = q.shape
    k, kts, khs, total, hkv, _ = _strided(k, layout)
    v, vts, vhs, _, _, _ = _strided(v, layout)
    cu = _c(cu, np.int32)
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    out = np.empty((b, hq, d), np.float64)
    lib().oracle_dense_attn(_p(q), _p(k), ctypes.c_int64(kts), ctypes.c_int64(khs), _p(v),
                            ctypes.c_int64(vts), ctypes.c_int64(vhs), _p(cu), b, hq, hkv, d,
                            ctypes.c_double(scale), _p(out))
    return out
