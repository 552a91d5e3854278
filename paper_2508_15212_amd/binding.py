"""ctypes binding of the C ABI declared in ``include/spark.h``.

Argument marshalling only: tensors are torch device tensors used as raw device memory
(``data_ptr()``), the stream is torch's current HIP stream.  There is no fallback: if the
shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libspark_hip.so")

PACK_BF16, PACK_INT8 = 0, 1
RECOVER_GAUSSIAN, RECOVER_EXPONENTIAL = 1, 2
OUT_BF16, OUT_F32 = 0, 1
ERR_MISMATCH = 5

EXPORTS = ["spark_packed_bytes", "spark_prune_workspace", "spark_decode_workspace", "spark_decode_workspace_init", "spark_decode_splits",
           "spark_prune", "spark_decode_attn", "spark_unpack", "spark_probe_read", "spark_status_string",
           "spark_packed_values_bytes", "spark_prune_values", "spark_unpack_values", "spark_decode_attn_values", "spark_decode_attn_tail",
           "spark_decode_attn_values_tail", "spark_decode_attn_sampled", "spark_unpack_stats", "spark_check_packed",
           "spark_decode_attn_static", "spark_packed_topp_bytes", "spark_prune_topp", "spark_decode_attn_topp",
           "spark_unpack_topp", "spark_decode_timeline"]


class SparkError(RuntimeError):
    pass


class SparkDesc(ctypes.Structure):
    """Mirror of ``struct spark_desc``."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("keep", ctypes.c_int32), ("window", ctypes.c_int32),
        ("pack_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("total_tokens", ctypes.c_int64),
        ("k_token_stride", ctypes.c_int64), ("k_head_stride", ctypes.c_int64),
        ("v_token_stride", ctypes.c_int64), ("v_head_stride", ctypes.c_int64),
        ("softmax_scale", ctypes.c_float), ("n_splits", ctypes.c_int32),
        ("keep_v", ctypes.c_int32), ("stats", ctypes.c_int32), ("tail_capacity", ctypes.c_int32),
        ("max_seqlen", ctypes.c_int32),
    ]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise SparkError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                         "(or paper_2508_15212_amd/build.py) first; there is no fallback path")
    lib = ctypes.CDLL(_LIB_PATH)
    dp = ctypes.POINTER(SparkDesc)
    vp = ctypes.c_void_p
    lib.spark_packed_bytes.restype = ctypes.c_size_t
    lib.spark_packed_bytes.argtypes = [dp]
    lib.spark_prune_workspace.restype = ctypes.c_size_t
    lib.spark_prune_workspace.argtypes = [dp]
    lib.spark_decode_workspace.restype = ctypes.c_size_t
    lib.spark_decode_workspace.argtypes = [dp]
    lib.spark_decode_workspace_init.restype = ctypes.c_int
    lib.spark_decode_workspace_init.argtypes = [dp, vp, ctypes.c_size_t, vp]
    lib.spark_decode_splits.restype = ctypes.c_int32
    lib.spark_decode_splits.argtypes = [dp]
    lib.spark_prune.restype = ctypes.c_int
    lib.spark_prune.argtypes = [dp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.spark_decode_attn.restype = ctypes.c_int
    lib.spark_decode_attn.argtypes = [dp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.spark_unpack.restype = ctypes.c_int
    lib.spark_unpack.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
    lib.spark_packed_values_bytes.restype = ctypes.c_size_t
    lib.spark_packed_values_bytes.argtypes = [dp]
    lib.spark_prune_values.restype = ctypes.c_int
    lib.spark_prune_values.argtypes = [dp, vp, vp, vp]
    lib.spark_decode_attn_values.restype = ctypes.c_int
    lib.spark_decode_attn_values.argtypes = [dp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.spark_decode_attn_tail.restype = ctypes.c_int
    lib.spark_decode_attn_tail.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.spark_decode_attn_values_tail.restype = ctypes.c_int
    lib.spark_decode_attn_values_tail.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.spark_decode_attn_sampled.restype = ctypes.c_int
    lib.spark_decode_attn_sampled.argtypes = [dp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, ctypes.c_int32,
                                              ctypes.c_uint64, vp]
    lib.spark_unpack_stats.restype = ctypes.c_int
    lib.spark_unpack_stats.argtypes = [dp, vp, vp, vp, vp]
    lib.spark_unpack_values.restype = ctypes.c_int
    lib.spark_unpack_values.argtypes = [dp, vp, vp, vp, vp]
    lib.spark_decode_attn_static.restype = ctypes.c_int
    lib.spark_decode_attn_static.argtypes = [dp, vp, vp, vp, vp, vp, vp]
    lib.spark_packed_topp_bytes.restype = ctypes.c_size_t
    lib.spark_packed_topp_bytes.argtypes = [dp]
    lib.spark_prune_topp.restype = ctypes.c_int
    lib.spark_prune_topp.argtypes = [dp, vp, vp, vp, ctypes.c_int32, vp, vp]
    lib.spark_decode_attn_topp.restype = ctypes.c_int
    lib.spark_decode_attn_topp.argtypes = [dp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.spark_unpack_topp.restype = ctypes.c_int
    lib.spark_unpack_topp.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
    lib.spark_check_packed.restype = ctypes.c_int
    lib.spark_check_packed.argtypes = [dp, vp, ctypes.c_int32, vp]
    lib.spark_probe_read.restype = ctypes.c_int
    lib.spark_probe_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int32, vp]
    lib.spark_decode_timeline.restype = ctypes.c_int
    lib.spark_decode_timeline.argtypes = [vp, ctypes.c_size_t]
    lib.spark_status_string.restype = ctypes.c_char_p
    lib.spark_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise SparkError(f"{what}: {load().spark_status_string(rc).decode()} (status {rc})")


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _ptr(t) -> int | None:
    return None if t is None else int(t.data_ptr())


def packed_bytes(desc: SparkDesc) -> int:
    return int(load().spark_packed_bytes(ctypes.byref(desc)))


def decode_workspace_bytes(desc: SparkDesc) -> int:
    return int(load().spark_decode_workspace(ctypes.byref(desc)))


def decode_workspace_init(desc: SparkDesc, workspace: torch.Tensor) -> None:
    rc = load().spark_decode_workspace_init(ctypes.byref(desc), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "spark_decode_workspace_init")


def new_decode_workspace(desc: SparkDesc) -> torch.Tensor:
    """Allocate (through torch) and prepare a workspace for spark_decode_attn."""
    ws = torch.empty(max(16, decode_workspace_bytes(desc)), dtype=torch.uint8, device="cuda")
    decode_workspace_init(desc, ws)
    return ws


def decode_splits(desc: SparkDesc) -> int:
    return int(load().spark_decode_splits(ctypes.byref(desc)))


def prune(desc: SparkDesc, k: torch.Tensor, qwin: torch.Tensor, cu: torch.Tensor,
          packed: torch.Tensor) -> None:
    """spark_prune: k, qwin bf16-bit tensors on the device; packed a uint8 buffer of packed_bytes()."""
    ws_bytes = int(load().spark_prune_workspace(ctypes.byref(desc)))
    assert ws_bytes == 0
    rc = load().spark_prune(ctypes.byref(desc), _ptr(k), _ptr(qwin), _ptr(cu), _ptr(packed), None, 0, _stream())
    _check(rc, "spark_prune")


def decode_attn(desc: SparkDesc, q: torch.Tensor, packed: torch.Tensor, v: torch.Tensor, cu: torch.Tensor,
                out: torch.Tensor, workspace: torch.Tensor) -> None:
    rc = load().spark_decode_attn(ctypes.byref(desc), _ptr(q), _ptr(packed), _ptr(v), _ptr(cu), _ptr(out),
                                  _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "spark_decode_attn")


STATIC_WORKSPACE_BYTES = 4 << 20


def decode_attn_static(desc: SparkDesc, q: torch.Tensor, packed: torch.Tensor, v: torch.Tensor, cu: torch.Tensor,
                       out: torch.Tensor) -> None:
    """spark_decode_attn_static: decode with the library's own per-GPU scratch array (no workspace argument)."""
    rc = load().spark_decode_attn_static(ctypes.byref(desc), _ptr(q), _ptr(packed), _ptr(v), _ptr(cu), _ptr(out),
                                         _stream())
    _check(rc, "spark_decode_attn_static")


def packed_topp_bytes(desc: SparkDesc) -> int:
    return int(load().spark_packed_topp_bytes(ctypes.byref(desc)))


def prune_topp(desc: SparkDesc, k: torch.Tensor, qwin: torch.Tensor, cu: torch.Tensor, p_basis_points: int,
               packed: torch.Tensor) -> None:
    """spark_prune_topp: the variant that keeps, per row, the fewest channels holding p of the row's saliency."""
    rc = load().spark_prune_topp(ctypes.byref(desc), _ptr(k), _ptr(qwin), _ptr(cu), int(p_basis_points), _ptr(packed),
                                 _stream())
    _check(rc, "spark_prune_topp")


def decode_attn_topp(desc: SparkDesc, q: torch.Tensor, packed: torch.Tensor, v: torch.Tensor, cu: torch.Tensor,
                     out: torch.Tensor, workspace: torch.Tensor) -> None:
    rc = load().spark_decode_attn_topp(ctypes.byref(desc), _ptr(q), _ptr(packed), _ptr(v), _ptr(cu), _ptr(out),
                                       _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "spark_decode_attn_topp")


def unpack_topp(desc: SparkDesc, packed: torch.Tensor, mask=None, count=None, vals=None, mu=None, a=None) -> None:
    rc = load().spark_unpack_topp(ctypes.byref(desc), _ptr(packed), _ptr(mask), _ptr(count), _ptr(vals), _ptr(mu),
                                  _ptr(a), _stream())
    _check(rc, "spark_unpack_topp")


def packed_values_bytes(desc: SparkDesc) -> int:
    return int(load().spark_packed_values_bytes(ctypes.byref(desc)))


def prune_values(desc: SparkDesc, v: torch.Tensor, packed_v: torch.Tensor) -> None:
    """spark_prune_values: v bf16-bit tensor on the device; packed_v a uint8 buffer of packed_values_bytes()."""
    rc = load().spark_prune_values(ctypes.byref(desc), _ptr(v), _ptr(packed_v), _stream())
    _check(rc, "spark_prune_values")


def decode_attn_values(desc: SparkDesc, q: torch.Tensor, packed: torch.Tensor, packed_v: torch.Tensor,
                       cu: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor) -> None:
    rc = load().spark_decode_attn_values(ctypes.byref(desc), _ptr(q), _ptr(packed), _ptr(packed_v), _ptr(cu),
                                         _ptr(out), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "spark_decode_attn_values")


def decode_attn_tail(desc: SparkDesc, q: torch.Tensor, packed: torch.Tensor, v: torch.Tensor, cu: torch.Tensor,
                     tail_k: torch.Tensor, tail_v: torch.Tensor, tail_len: torch.Tensor, out: torch.Tensor,
                     workspace: torch.Tensor) -> None:
    rc = load().spark_decode_attn_tail(ctypes.byref(desc), _ptr(q), _ptr(packed), _ptr(v), _ptr(cu), _ptr(tail_k),
                                       _ptr(tail_v), _ptr(tail_len), _ptr(out), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "spark_decode_attn_tail")


def decode_attn_values_tail(desc: SparkDesc, q: torch.Tensor, packed: torch.Tensor, packed_v: torch.Tensor,
                            cu: torch.Tensor, tail_k: torch.Tensor, tail_v: torch.Tensor, tail_len: torch.Tensor,
                            out: torch.Tensor, workspace: torch.Tensor) -> None:
    rc = load().spark_decode_attn_values_tail(ctypes.byref(desc), _ptr(q), _ptr(packed), _ptr(packed_v), _ptr(cu),
                                              _ptr(tail_k), _ptr(tail_v), _ptr(tail_len), _ptr(out), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(), _stream())
    _check(rc, "spark_decode_attn_values_tail")


def decode_attn_sampled(desc: SparkDesc, q: torch.Tensor, packed: torch.Tensor, v: torch.Tensor, cu: torch.Tensor,
                        out: torch.Tensor, workspace: torch.Tensor, recovery: int, seed: int) -> None:
    rc = load().spark_decode_attn_sampled(ctypes.byref(desc), _ptr(q), _ptr(packed), _ptr(v), _ptr(cu), _ptr(out),
                                          _ptr(workspace), workspace.numel() * workspace.element_size(),
                                          int(recovery), ctypes.c_uint64(seed & 0xFFFFFFFFFFFFFFFF), _stream())
    _check(rc, "spark_decode_attn_sampled")


def unpack_stats(desc: SparkDesc, packed: torch.Tensor, mu_all=None, sigma=None) -> None:
    rc = load().spark_unpack_stats(ctypes.byref(desc), _ptr(packed), _ptr(mu_all), _ptr(sigma), _stream())
    _check(rc, "spark_unpack_stats")


def unpack_values(desc: SparkDesc, packed_v: torch.Tensor, mask=None, vals=None) -> None:
    rc = load().spark_unpack_values(ctypes.byref(desc), _ptr(packed_v), _ptr(mask), _ptr(vals), _stream())
    _check(rc, "spark_unpack_values")


def unpack(desc: SparkDesc, packed: torch.Tensor, mask=None, vals=None, mu=None, scale=None, a=None) -> None:
    rc = load().spark_unpack(ctypes.byref(desc), _ptr(packed), _ptr(mask), _ptr(vals), _ptr(mu), _ptr(scale),
                             _ptr(a), _stream())
    _check(rc, "spark_unpack")


def check_packed(desc: SparkDesc, packed: torch.Tensor, is_value_cache: bool = False) -> int:
    """spark_check_packed: status code (0 = the cache matches the description, 5 = mismatch); synchronises."""
    rc = int(load().spark_check_packed(ctypes.byref(desc), _ptr(packed), 1 if is_value_cache else 0, _stream()))
    if rc not in (0, ERR_MISMATCH):
        _check(rc, "spark_check_packed")
    return rc


def decode_timeline(buffer) -> None:
    """spark_decode_timeline (include/spark_bench.h): later decode launches file eight int64 words per block into
    `buffer` (an int64 device tensor the caller keeps alive); None switches the aid off."""
    if buffer is None:
        rc = load().spark_decode_timeline(None, 0)
    else:
        rc = load().spark_decode_timeline(_ptr(buffer), buffer.numel() * buffer.element_size())
    _check(rc, "spark_decode_timeline")


def probe_read(src: torch.Tensor, sink: torch.Tensor, n_blocks: int) -> None:
    """spark_probe_read (include/spark_bench.h): stream `src` once (measurement aid)."""
    rc = load().spark_probe_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), n_blocks, _stream())
    _check(rc, "spark_probe_read")
