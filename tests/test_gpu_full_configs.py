"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration the
library picks by itself (the one bench.py times).  The CPU oracle is fast enough (seconds on the host
cores) to check every row and every output element, so nothing is sampled:

    masks, kept entries / int8 codes, scales, a  : bit-exact
    mu                                           : 1e-5 relative
    decode output (float32 out)                  : max |err| <= 1e-2, mean |err| <= 1e-3

Near-tie rows (relative saliency gap < 1e-6 at the cut) are counted and printed.
"""
import functools

import numpy as np
import pytest

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import run_gpu_case

pytestmark = pytest.mark.gpu


@functools.lru_cache(maxsize=1)
def _tensors(idx):
    w = wl.config(idx)
    return w, wl.generate(w)


def _check(w, t, int8=False, decode=True):
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    if int8:
        pr = oracle.quant_int8(pr)
    res = run_gpu_case(w, t, pack=spark.PACK_INT8 if int8 else spark.PACK_BF16, want_bf16=False)
    rows = w.total * w.n_kv_heads
    print(f"{w.name} T={w.keep} int8={int8}: rows={rows} near-ties(<1e-6)={pr.near_ties()} "
          f"splits={spark.decode_splits(res['desc'])}")
    assert np.array_equal(res["a"], a32)
    assert np.array_equal(res["mask"], pr.mask), "kept-channel sets differ"
    if int8:
        assert np.array_equal(res["scale"], pr.scale) and np.array_equal(res["vals"], pr.codes)
    else:
        assert np.array_equal(res["vals"], pr.kept)
    assert np.allclose(res["mu"], pr.mu32, rtol=1e-5, atol=1e-30)
    if decode:
        ref = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
        err = np.abs(res["out_f32"].astype(np.float64) - ref)
        print(f"   decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
        assert err.max() <= 1e-2 and err.mean() <= 1e-3


def test_config2_llama8b_32k_keep26():
    w, t = _tensors(2)
    _check(w, t)


def test_config2_keep25_paper_floor():
    """T = floor((1 - 0.8) * 128) = 25, the paper's own rounding of an 80 % pruning ratio."""
    w, t = _tensors(2)
    w2 = wl.config(2, keep=25)
    _check(w2, t)


@pytest.mark.parametrize("T", [64, 38, 26])
def test_config3_prune_131k(T):
    w, t = _tensors(3)
    _check(wl.config(3, keep=T), t, decode=False)


def test_config4_ragged_batch64_keep64():
    w, t = _tensors(4)
    _check(w, t)


@pytest.mark.parametrize("int8", [False, True])
def test_config5_qwen32b_131k(int8):
    w, t = _tensors(5)
    _check(w, t, int8=int8)


def test_config2_pruned_values_keep64():
    """Keys at T = 26 and values at T_v = 64 (the appendix's joint pruning), every row and output checked."""
    import torch
    from tests.gpu_util import make_desc, to_dev
    w, t = _tensors(2)
    Tv = 64
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    pv = oracle.prune_values(t.v, t.layout, Tv)
    ref = oracle.decode_literal(t.q, pr, oracle.expand_values(pv), "NHD", t.cu)
    desc = make_desc(w)
    desc.keep_v = Tv
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(spark.packed_bytes(desc), dtype=torch.uint8, device="cuda")
    packed_v = torch.empty(spark.packed_values_bytes(desc), dtype=torch.uint8, device="cuda")
    dv = to_dev(t.v)
    spark.prune(desc, to_dev(t.k), to_dev(t.qwin), dcu, packed)
    spark.prune_values(desc, dv, packed_v)
    del dv
    mask = torch.empty((w.total, w.n_kv_heads, 4), dtype=torch.int32, device="cuda")
    vals = torch.empty((w.total, w.n_kv_heads, Tv), dtype=torch.int16, device="cuda")
    spark.unpack_values(desc, packed_v, mask, vals)
    print(f"{w.name} Tv={Tv}: value near-ties(<1e-6)={pv.near_ties()} of {pv.gap.size}")
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), pv.mask), "kept value-channel sets differ"
    assert np.array_equal(vals.cpu().numpy().view(np.uint16), pv.kept)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn_values(desc, to_dev(t.q), packed, packed_v, dcu, out, spark.new_decode_workspace(desc))
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    print(f"   decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert err.max() <= 1e-2 and err.mean() <= 1e-3


def test_config2_with_128_appended_rows():
    import torch
    from tests.gpu_util import make_desc, to_dev
    w, t = _tensors(2)
    cap = 128
    rng = np.random.default_rng(5)
    shape = (w.batch, cap, w.n_kv_heads, w.head_dim)
    tk = wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    tv = wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    tl = rng.integers(1, cap + 1, size=w.batch).astype(np.int32)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    ref = oracle.decode_literal_tail(t.q, pr, t.v, t.layout, t.cu, tk, tv, tl)
    desc = make_desc(w)
    desc.tail_capacity = cap
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(spark.packed_bytes(desc), dtype=torch.uint8, device="cuda")
    spark.prune(desc, to_dev(t.k), to_dev(t.qwin), dcu, packed)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn_tail(desc, to_dev(t.q), packed, to_dev(t.v), dcu, to_dev(tk), to_dev(tv),
                           torch.from_numpy(tl).cuda(), out, spark.new_decode_workspace(desc))
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    print(f"{w.name} + appended rows {tl.tolist()}: decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert err.max() <= 1e-2 and err.mean() <= 1e-3


@pytest.mark.parametrize("kind", [spark.RECOVER_GAUSSIAN, spark.RECOVER_EXPONENTIAL])
def test_config2_sampled_recovery(kind):
    """The sampled recovery functions at the 32K benchmark shape: statistics rows (mean and standard deviation of
    every row's saliencies to 1e-5), masks bit-exact, decode against the oracle's draw of the same seed."""
    import torch
    from tests.gpu_util import make_desc, to_dev
    w, t = _tensors(2)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    mu, sigma = oracle.row_stats(t.k, t.layout, a32, t.cu)
    desc = make_desc(w)
    desc.stats = 1
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(spark.packed_bytes(desc), dtype=torch.uint8, device="cuda")
    spark.prune(desc, to_dev(t.k), to_dev(t.qwin), dcu, packed)
    mask = torch.empty((w.total, w.n_kv_heads, 4), dtype=torch.int32, device="cuda")
    mua = torch.empty((w.total, w.n_kv_heads), dtype=torch.float32, device="cuda")
    sg = torch.empty_like(mua)
    spark.unpack(desc, packed, mask, None, None, None, None)
    spark.unpack_stats(desc, packed, mua, sg)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), pr.mask)
    assert np.allclose(mua.cpu().numpy(), mu, rtol=1e-5, atol=1e-30)
    assert np.allclose(sg.cpu().numpy(), sigma, rtol=1e-5, atol=1e-6 * np.abs(mu).max())
    del mask, mua, sg
    seed = 0x5EED00000000 + kind
    ref = oracle.decode_sampled(kind, seed, t.q, pr, mu, sigma, t.v, t.layout, t.cu)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn_sampled(desc, to_dev(t.q), packed, to_dev(t.v), dcu, out, spark.new_decode_workspace(desc), kind, seed)
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    print(f"{w.name} sampled recovery {kind}: decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert err.max() <= 1e-2 and err.mean() <= 1e-3


def test_config2_decode_replayed_500_times_on_one_workspace():
    """The split merge (partial states written with device-scope stores, counted at an arrival counter, folded by the
    block that arrives last) replayed on ONE workspace: 500 launches rotating over four query sets, every output
    compared bit for bit with the first output of the same query set; stops at the first mismatch."""
    import torch
    from tests.gpu_util import make_desc, to_dev
    w, t = _tensors(2)
    desc = make_desc(w, out_dtype=spark.OUT_F32)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(spark.packed_bytes(desc), dtype=torch.uint8, device="cuda")
    spark.prune(desc, to_dev(t.k), to_dev(t.qwin), dcu, packed)
    dv = to_dev(t.v)
    rng = np.random.default_rng(9)
    qs = [to_dev(t.q)] + [to_dev(wl.f32_to_bf16_bits(rng.standard_normal(t.q.shape).astype(np.float32))) for _ in range(3)]
    ws = spark.new_decode_workspace(desc)
    first = [None] * len(qs)
    outs = [torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda") for _ in range(8)]
    for i in range(500):
        j = i % len(qs)
        o = outs[i % len(outs)]
        spark.decode_attn(desc, qs[j], packed, dv, dcu, o, ws)
        if first[j] is None:
            first[j] = o.clone()
        elif i % 8 == 7 or i == 499:      # (check in groups so that launches really run back to back)
            for back in range(min(8, i + 1)):
                ii = i - back
                assert torch.equal(outs[ii % len(outs)], first[ii % len(qs)]), f"replay {ii} differs from its first run"
    torch.cuda.synchronize()
    ref = oracle.decode_literal(t.q, oracle.prune(t.k, t.layout, oracle.window_stat(t.qwin, w.n_kv_heads)[2], t.cu, w.keep),
                                t.v, t.layout, t.cu)
    assert np.abs(first[0].cpu().numpy().astype(np.float64) - ref).max() <= 1e-2


def test_config4_balanced_decode_replayed_400_times_on_one_workspace():
    """The same soak for the balanced cut of the ragged batch, where wavefronts (2048 of them) count in one by one
    and any of them may be the one that merges a pair: 400 launches on one workspace, rotating query sets, every
    output bit for bit equal to the first output of its query set (the merge folds the partials in slot order,
    whatever the order of arrival)."""
    import torch
    from tests.gpu_util import make_desc, to_dev
    w, t = _tensors(4)
    desc = make_desc(w, out_dtype=spark.OUT_F32)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(spark.packed_bytes(desc), dtype=torch.uint8, device="cuda")
    spark.prune(desc, to_dev(t.k), to_dev(t.qwin), dcu, packed)
    dv = to_dev(t.v)
    rng = np.random.default_rng(11)
    qs = [to_dev(t.q)] + [to_dev(wl.f32_to_bf16_bits(rng.standard_normal(t.q.shape).astype(np.float32))) for _ in range(3)]
    # (the library's own choice for this batch: more partial slots than one block per sequence would need)
    assert spark.decode_workspace_bytes(desc) > spark.decode_workspace_bytes(make_desc(w, out_dtype=spark.OUT_F32, n_splits=1))
    ws = spark.new_decode_workspace(desc)
    first = [None] * len(qs)
    outs = [torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda") for _ in range(8)]
    for i in range(400):
        j = i % len(qs)
        o = outs[i % len(outs)]
        spark.decode_attn(desc, qs[j], packed, dv, dcu, o, ws)
        if first[j] is None:
            first[j] = o.clone()
        elif i % 8 == 7 or i == 399:
            for back in range(min(8, i + 1)):
                ii = i - back
                assert torch.equal(outs[ii % len(outs)], first[ii % len(qs)]), f"replay {ii} differs from its first run"
    torch.cuda.synchronize()
    ref = oracle.decode_literal(t.q, oracle.prune(t.k, t.layout, oracle.window_stat(t.qwin, w.n_kv_heads)[2], t.cu, w.keep),
                                t.v, t.layout, t.cu)
    assert np.abs(first[0].cpu().numpy().astype(np.float64) - ref).max() <= 1e-2


def test_config5_int8_keys_with_pruned_values_keep64():
    """The Qwen-shaped workload with int8 key entries and the value cache pruned to 64 channels per row."""
    import torch
    from tests.gpu_util import make_desc, to_dev
    w, t = _tensors(5)
    Tv = 64
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.quant_int8(oracle.prune(t.k, t.layout, a32, t.cu, w.keep))
    pv = oracle.prune_values(t.v, t.layout, Tv)
    ref = oracle.decode_literal(t.q, pr, oracle.expand_values(pv), "NHD", t.cu)
    desc = make_desc(w, pack=spark.PACK_INT8)
    desc.keep_v = Tv
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(spark.packed_bytes(desc), dtype=torch.uint8, device="cuda")
    packed_v = torch.empty(spark.packed_values_bytes(desc), dtype=torch.uint8, device="cuda")
    dv = to_dev(t.v)
    spark.prune(desc, to_dev(t.k), to_dev(t.qwin), dcu, packed)
    spark.prune_values(desc, dv, packed_v)
    del dv
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn_values(desc, to_dev(t.q), packed, packed_v, dcu, out, spark.new_decode_workspace(desc))
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    print(f"{w.name} int8 keys + Tv={Tv}: decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert err.max() <= 1e-2 and err.mean() <= 1e-3
