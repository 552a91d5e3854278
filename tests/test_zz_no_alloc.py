"""spark_decode_attn_static (the entry point that allocates nothing) against spark_decode_attn, through the
C ABI: same inputs, same outputs, on two calls in a row, the second over a smaller batch -- the per-GPU
scratch array still holds the first call's partial states and must not leak them into the second."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import run_gpu_case

pytestmark = pytest.mark.gpu


def _case(w):
    t = wl.generate(w)
    res = run_gpu_case(w, t, want_unpack=False, want_bf16=False)     # spark_prune + spark_decode_attn
    desc = res["desc"]
    assert spark.decode_workspace_bytes(desc) <= spark.STATIC_WORKSPACE_BYTES
    dk, dv, dqw, dq, dcu = res["dev"]
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
    spark.decode_attn_static(desc, dq, res["packed"], dv, dcu, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got))
    assert np.array_equal(got, res["out_f32"]), "static-scratch decode differs from the workspace decode"
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    err = np.abs(got.astype(np.float64) - oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu))
    assert err.max() <= 1e-2 and err.mean() <= 1e-3


def test_static_scratch_decode_two_calls_second_smaller():
    _case(wl.small(name="static_big", batch=3, n_q_heads=16, n_kv_heads=4, seqlens=(9000, 4100, 700), seed=81))
    _case(wl.small(name="static_small", batch=2, n_q_heads=16, n_kv_heads=4, seqlens=(300, 150), seed=82))
    _case(wl.small(name="static_big", batch=3, n_q_heads=16, n_kv_heads=4, seqlens=(9000, 4100, 700), seed=81))


def test_static_scratch_uses_the_cut_by_length_where_the_balanced_cut_does_not_fit():
    """64 short sequences x 8 KV heads: spark_decode_attn takes the balanced cut, whose partial slots exceed the
    array; the cut by length fits, and the static entry point uses that one (same result up to summation order)."""
    rng = np.random.default_rng(83)
    lens = tuple(int(x) for x in rng.integers(300, 1000, size=64))        # (enough tiles for the balanced cut)
    w = wl.small(name="static_ragged", batch=64, n_q_heads=32, n_kv_heads=8, keep=26, seqlens=lens, seed=83)
    t = wl.generate(w)
    res = run_gpu_case(w, t, want_unpack=False, want_bf16=False)
    desc = res["desc"]
    assert spark.decode_workspace_bytes(desc) > spark.STATIC_WORKSPACE_BYTES
    dk, dv, dqw, dq, dcu = res["dev"]
    for _ in range(2):
        out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        spark.decode_attn_static(desc, dq, res["packed"], dv, dcu, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.all(np.isfinite(got))
        assert np.abs(got - res["out_f32"]).max() <= 1e-4
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    err = np.abs(got.astype(np.float64) - oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu))
    assert err.max() <= 1e-2 and err.mean() <= 1e-3


def test_static_scratch_rejects_what_does_not_fit():
    d = spark.SparkDesc(batch=4096, n_q_heads=64, n_kv_heads=8, head_dim=128, keep=26, window=32,
                        total_tokens=4096 * 64, k_token_stride=128, k_head_stride=128 * 4096 * 64,
                        v_token_stride=128, v_head_stride=128 * 4096 * 64)
    assert spark.decode_workspace_bytes(d) > spark.STATIC_WORKSPACE_BYTES
    A = 0x7F0000000000
    import ctypes
    assert spark.load().spark_decode_attn_static(ctypes.byref(d), A, A, A, A, A, None) == 3
