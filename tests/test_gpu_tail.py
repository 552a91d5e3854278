"""GPU parity for decode with appended, never-pruned rows (the dense tail): the pruned prefix and the
appended rows share one softmax.  Tolerance as for plain decode: max |err| <= 1e-2, mean |err| <= 1e-3."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import make_desc, to_dev

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 1e-2, 1e-3


def _tail_case(w, cap, tail_len, seed, n_splits=0, scale_k=1.0):
    t = wl.generate(w)
    rng = np.random.default_rng(seed)
    shape = (w.batch, cap, w.n_kv_heads, w.head_dim)
    tk = wl.f32_to_bf16_bits((rng.standard_normal(shape) * scale_k).astype(np.float32))
    tv = wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    tl = np.asarray(tail_len, np.int32)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    ref = oracle.decode_literal_tail(t.q, pr, t.v, t.layout, t.cu, tk, tv, tl)

    desc = make_desc(w, n_splits=n_splits)
    desc.tail_capacity = cap
    dk, dv, dqw, dq = to_dev(t.k), to_dev(t.v), to_dev(t.qwin), to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(max(spark.packed_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    spark.prune(desc, dk, dqw, dcu, packed)
    ws = spark.new_decode_workspace(desc)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn_tail(desc, dq, packed, dv, dcu, to_dev(tk), to_dev(tv), torch.from_numpy(tl).cuda(), out, ws)
    # the same workspace serves a plain decode afterwards (the spare slot is simply not read)
    out_plain = torch.empty_like(out)
    spark.decode_attn(desc, dq, packed, dv, dcu, out_plain, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    err = np.abs(got.astype(np.float64) - ref)
    print(f"{w.name}: tail decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert np.all(np.isfinite(got))
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS
    plain_ref = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    assert np.abs(out_plain.cpu().numpy() - plain_ref).max() <= MAX_ABS
    return got, ref


@pytest.mark.parametrize("G,Hkv", [(1, 2), (2, 2), (4, 2), (8, 2), (16, 1)])
def test_tail_group_sizes(G, Hkv):
    w = wl.small(name=f"tail_gqa{G}", n_q_heads=G * Hkv, n_kv_heads=Hkv, keep=26, seqlens=(257, 64, 190), batch=3,
                 seed=400 + G)
    _tail_case(w, cap=70, tail_len=(70, 0, 33), seed=400 + G)


def test_tail_longer_than_one_chunk_and_many_splits():
    w = wl.small(name="tail_long", batch=2, seqlens=(1500, 700), keep=26, seed=410)
    _tail_case(w, cap=600, tail_len=(600, 257), seed=410, n_splits=7)


def test_tail_dominates_the_softmax():
    """Appended keys ten times larger: nearly all probability mass sits on the appended rows."""
    w = wl.small(name="tail_peaked", batch=2, seqlens=(300, 141), keep=64, seed=420)
    _tail_case(w, cap=16, tail_len=(16, 3), seed=420, scale_k=10.0)


def test_tail_with_empty_prefix_and_empty_tail():
    w = wl.small(name="tail_edges", batch=6, seqlens=(0, 1, 63, 64, 65, 0), keep=26, seed=430)
    got, _ = _tail_case(w, cap=8, tail_len=(5, 0, 8, 1, 0, 0), seed=430)
    assert np.all(got[5] == 0)          # neither prefix nor appended rows: zero output


def test_tail_together_with_pruned_values():
    """Packed keys + packed values + appended dense rows in one call."""
    w = wl.small(name="tail_kv", batch=3, n_q_heads=8, n_kv_heads=2, keep=26, seqlens=(257, 64, 190), seed=440)
    t = wl.generate(w)
    cap, Tv = 40, 64
    rng = np.random.default_rng(440)
    shape = (w.batch, cap, w.n_kv_heads, w.head_dim)
    tk = wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    tv = wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    tl = np.asarray((40, 7, 0), np.int32)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    pv = oracle.prune_values(t.v, t.layout, Tv)
    ref = oracle.decode_literal_tail(t.q, pr, oracle.expand_values(pv), "NHD", t.cu, tk, tv, tl)
    desc = make_desc(w)
    desc.keep_v, desc.tail_capacity = Tv, cap
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(max(spark.packed_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    packed_v = torch.empty(max(spark.packed_values_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    spark.prune(desc, to_dev(t.k), to_dev(t.qwin), dcu, packed)
    spark.prune_values(desc, to_dev(t.v), packed_v)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn_values_tail(desc, to_dev(t.q), packed, packed_v, dcu, to_dev(tk), to_dev(tv),
                                  torch.from_numpy(tl).cuda(), out, spark.new_decode_workspace(desc))
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    print(f"tail + pruned values: max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS
