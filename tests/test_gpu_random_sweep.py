"""Seeded sweep over random small problem shapes: group size, head count, kept channels, ragged lengths
(empty sequences included), layout, forced or library-chosen blocks per sequence, optional value pruning,
optional appended rows, optional statistics rows with a sampled recovery function, each checked against the CPU oracle (masks and kept entries bit for bit,
decode output max |err| <= 1e-2, mean |err| <= 1e-3)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import make_desc, to_dev

pytestmark = pytest.mark.gpu


def _one_case(rng, idx, int8=False):
    G = int(rng.choice([1, 2, 4, 8, 16]))
    hkv = int(rng.integers(1, 4))
    batch = int(rng.integers(1, 6))
    lens = tuple(int(x) for x in rng.choice([0, 1, 5, 63, 64, 65, 127, 130, 300, 777], size=batch))
    T = int(rng.choice([1, 13, 25, 26, 38, 64, 100, 128]))
    layout = str(rng.choice(["HND", "NHD"]))
    n_splits = int(rng.choice([0, 0, 1, 2, 5, -1, -1]))      # (-1: the balanced cut where the entry point has one)
    Tv = int(rng.choice([0, 0, 26, 38, 64, 90]))
    cap = int(rng.choice([0, 0, 3, 70, 300]))
    stats = int(rng.choice([0, 0, 1]))            # rows that also carry the all-channel mean / standard deviation
    rec = int(rng.choice([0, 1, 2])) if (stats and not Tv and not cap) else 0
    w = wl.small(name=f"sweep{idx}", batch=batch, n_q_heads=G * hkv, n_kv_heads=hkv, keep=T, seqlens=lens,
                 seed=1000 + idx)
    t = wl.generate(w)
    tag = (f"case {idx}: G={G} Hkv={hkv} lens={lens} T={T} {layout} splits={n_splits} Tv={Tv} cap={cap} "
           f"stats={stats} rec={rec} int8={int(int8)}")
    print(tag, flush=True)
    _, _, a32 = oracle.window_stat(t.qwin, hkv)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, T)
    if int8:
        pr = oracle.quant_int8(pr)
    v_for_oracle, v_layout = t.v, t.layout
    if Tv:
        pv = oracle.prune_values(t.v, t.layout, Tv)
        v_for_oracle, v_layout = oracle.expand_values(pv), "NHD"
    if rec:
        mu_all, sigma_all = oracle.row_stats(t.k, t.layout, a32, t.cu)
        ref = oracle.decode_sampled(rec, 77 + idx, t.q, pr, mu_all, sigma_all, t.v, t.layout, t.cu)
    elif cap:
        tk = wl.f32_to_bf16_bits(rng.standard_normal((batch, cap, hkv, 128)).astype(np.float32))
        tv = wl.f32_to_bf16_bits(rng.standard_normal((batch, cap, hkv, 128)).astype(np.float32))
        tl = rng.integers(0, cap + 1, size=batch).astype(np.int32)
        ref = oracle.decode_literal_tail(t.q, pr, v_for_oracle, v_layout, t.cu, tk, tv, tl)
    else:
        ref = oracle.decode_literal(t.q, pr, v_for_oracle, v_layout, t.cu)

    k, v = t.k, t.v
    if layout == "NHD":
        k = np.ascontiguousarray(k.transpose(1, 0, 2))
        v = np.ascontiguousarray(v.transpose(1, 0, 2))
    desc = make_desc(w, layout, pack=spark.PACK_INT8 if int8 else spark.PACK_BF16, n_splits=n_splits)
    desc.keep_v, desc.tail_capacity, desc.stats = Tv, cap, stats
    if w.total == 0:                       # no rows: any valid stride
        desc.k_head_stride = desc.v_head_stride = desc.k_token_stride = desc.v_token_stride = 128
    dk = to_dev(k) if w.total else torch.zeros(256, dtype=torch.int16, device="cuda")
    dv = to_dev(v) if w.total else torch.zeros(256, dtype=torch.int16, device="cuda")
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(max(spark.packed_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    spark.prune(desc, dk, to_dev(t.qwin), dcu, packed)
    if w.total:
        mask = torch.empty((w.total, hkv, 4), dtype=torch.int32, device="cuda")
        vals = torch.empty((w.total, hkv, T), dtype=torch.int8 if int8 else torch.int16, device="cuda")
        spark.unpack(desc, packed, mask, vals, None, None, None)
        assert np.array_equal(mask.cpu().numpy().view(np.uint32), pr.mask), tag
        if int8:
            assert np.array_equal(vals.cpu().numpy(), pr.codes), tag
        else:
            assert np.array_equal(vals.cpu().numpy().view(np.uint16), pr.kept), tag
    ws = spark.new_decode_workspace(desc)
    out = torch.full((batch, G * hkv, 128), float("nan"), dtype=torch.float32, device="cuda")
    dq = to_dev(t.q)
    if Tv:
        packed_v = torch.empty(max(spark.packed_values_bytes(desc), 256), dtype=torch.uint8, device="cuda")
        spark.prune_values(desc, dv, packed_v)
        if w.total:
            mv = torch.empty((w.total, hkv, 4), dtype=torch.int32, device="cuda")
            spark.unpack_values(desc, packed_v, mv, None)
            assert np.array_equal(mv.cpu().numpy().view(np.uint32), pv.mask), tag
        if cap:
            spark.decode_attn_values_tail(desc, dq, packed, packed_v, dcu, to_dev(tk), to_dev(tv),
                                          torch.from_numpy(tl).cuda(), out, ws)
        else:
            spark.decode_attn_values(desc, dq, packed, packed_v, dcu, out, ws)
    elif rec:
        spark.decode_attn_sampled(desc, dq, packed, dv, dcu, out, ws, rec, 77 + idx)
    elif cap:
        spark.decode_attn_tail(desc, dq, packed, dv, dcu, to_dev(tk), to_dev(tv), torch.from_numpy(tl).cuda(), out, ws)
    else:
        spark.decode_attn(desc, dq, packed, dv, dcu, out, ws)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.all(np.isfinite(got)), tag
    err = np.abs(got.astype(np.float64) - ref)
    assert err.max() <= 1e-2 and err.mean() <= 1e-3, (tag, err.max(), err.mean())


def test_random_shapes_against_the_oracle():
    rng = np.random.default_rng(20250815)
    for idx in range(240):
        _one_case(rng, idx)


def test_random_shapes_with_int8_key_storage():
    """The same sweep with the kept key entries stored as int8 codes (also together with pruned values and with
    appended rows)."""
    rng = np.random.default_rng(20250816)
    for idx in range(80):
        _one_case(rng, 5000 + idx, int8=True)
