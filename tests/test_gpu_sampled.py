"""GPU parity for the sampled recovery functions (Gaussian, Exponential): the cache written with
desc.stats = 1 carries the all-channel mean and standard deviation of each row's saliencies (compared to
1e-5 relative, absolute 1e-6 of the mean for the spread of near-constant rows); decode with the same seed
draws the same uniforms on both sides (integer hash), so outputs agree to the decode tolerance."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import make_desc, to_dev

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 1e-2, 1e-3


def _setup(w, t=None, layout="HND"):
    t = wl.generate(w) if t is None else t
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    mu, sigma = oracle.row_stats(t.k, t.layout, a32, t.cu)
    k, v = t.k, t.v
    if layout == "NHD":
        k = np.ascontiguousarray(k.transpose(1, 0, 2))
        v = np.ascontiguousarray(v.transpose(1, 0, 2))
    desc = make_desc(w, layout)
    desc.stats = 1
    dk, dv, dq = to_dev(k), to_dev(v), to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(max(spark.packed_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    spark.prune(desc, dk, to_dev(t.qwin), dcu, packed)
    return t, pr, mu, sigma, desc, packed, dv, dq, dcu


def _check_stats(w, pr, mu, sigma, desc, packed):
    mask = torch.empty((w.total, w.n_kv_heads, 4), dtype=torch.int32, device="cuda")
    vals = torch.empty((w.total, w.n_kv_heads, w.keep), dtype=torch.int16, device="cuda")
    mup = torch.empty((w.total, w.n_kv_heads), dtype=torch.float32, device="cuda")
    mua, sg = torch.empty_like(mup), torch.empty_like(mup)
    spark.unpack(desc, packed, mask, vals, mup, None, None)
    spark.unpack_stats(desc, packed, mua, sg)
    torch.cuda.synchronize()
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), pr.mask)
    assert np.array_equal(vals.cpu().numpy().view(np.uint16), pr.kept)
    assert np.allclose(mup.cpu().numpy(), pr.mu32, rtol=1e-5, atol=1e-30)
    assert np.allclose(mua.cpu().numpy(), mu, rtol=1e-5, atol=1e-30)
    assert np.allclose(sg.cpu().numpy(), sigma, rtol=1e-5, atol=1e-6 * np.abs(mu).max())


@pytest.mark.parametrize("T", [26, 64, 38, 127])
def test_row_statistics_and_selection_with_stats_rows(T):
    w = wl.small(name=f"stats{T}", keep=T, seqlens=(130, 321), seed=600 + T)
    t, pr, mu, sigma, desc, packed, dv, dq, dcu = _setup(w)
    _check_stats(w, pr, mu, sigma, desc, packed)
    # the degenerate recovery still works on such a cache (any-length kernel)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn(desc, dq, packed, dv, dcu, out, spark.new_decode_workspace(desc))
    ref = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    assert np.abs(out.cpu().numpy() - ref).max() <= MAX_ABS
    # ... also with the balanced cut (wavefronts on their own ranges of tiles)
    desc.n_splits = -1
    out2 = torch.empty_like(out)
    spark.decode_attn(desc, dq, packed, dv, dcu, out2, spark.new_decode_workspace(desc))
    assert np.abs(out2.cpu().numpy() - ref).max() <= MAX_ABS


@pytest.mark.parametrize("kind", [spark.RECOVER_GAUSSIAN, spark.RECOVER_EXPONENTIAL])
@pytest.mark.parametrize("G,Hkv,layout", [(1, 2, "HND"), (4, 2, "NHD"), (8, 2, "HND"), (16, 1, "HND")])
def test_sampled_decode_matches_oracle(kind, G, Hkv, layout):
    w = wl.small(name=f"sampled{kind}_{G}", batch=3, n_q_heads=G * Hkv, n_kv_heads=Hkv, keep=26,
                 seqlens=(257, 0, 190), seed=620 + G)
    t, pr, mu, sigma, desc, packed, dv, dq, dcu = _setup(w, layout=layout)
    _check_stats(w, pr, mu, sigma, desc, packed)
    seed = 0x1234567890ABCDEF + G
    ref = oracle.decode_sampled(kind, seed, t.q, pr, mu, sigma, t.v, t.layout, t.cu)
    ws = spark.new_decode_workspace(desc)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn_sampled(desc, dq, packed, dv, dcu, out, ws, kind, seed)
    out2 = torch.empty_like(out)
    spark.decode_attn_sampled(desc, dq, packed, dv, dcu, out2, ws, kind, seed + 1)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    err = np.abs(got.astype(np.float64) - ref)
    print(f"{w.name}: sampled decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert np.all(np.isfinite(got)) and np.all(got[1] == 0)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS
    # another seed is another draw: different from the first, and equal to the oracle's for that seed
    ref2 = oracle.decode_sampled(kind, seed + 1, t.q, pr, mu, sigma, t.v, t.layout, t.cu)
    assert np.abs(out2.cpu().numpy() - ref2).max() <= MAX_ABS
    assert np.abs(ref2 - ref).max() > 1e-4


def test_sampled_decode_many_splits_and_ragged_tiles():
    w = wl.small(name="sampled_splits", batch=2, seqlens=(1500, 700), keep=38, seed=640)
    t, pr, mu, sigma, desc, packed, dv, dq, dcu = _setup(w)
    desc.n_splits = 7
    ref = oracle.decode_sampled(oracle.GAUSSIAN, 11, t.q, pr, mu, sigma, t.v, t.layout, t.cu)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn_sampled(desc, dq, packed, dv, dcu, out, spark.new_decode_workspace(desc),
                              spark.RECOVER_GAUSSIAN, 11)
    assert np.abs(out.cpu().numpy() - ref).max() <= MAX_ABS


@pytest.mark.parametrize("kind", [spark.RECOVER_GAUSSIAN, spark.RECOVER_EXPONENTIAL])
@pytest.mark.parametrize("G,Hkv,T", [(4, 2, 26), (8, 1, 64), (1, 2, 37)])
def test_int8_storage_with_statistics_rows(kind, G, Hkv, T):
    """int8 codes and a statistics-carrying row together: codes, scales, masks bit-exact, the statistics those of
    the saliencies before quantisation, sampled and degenerate decode against the oracle over code * scale."""
    w = wl.small(name=f"i8stats{kind}_{G}_{T}", batch=3, n_q_heads=G * Hkv, n_kv_heads=Hkv, keep=T,
                 seqlens=(300, 0, 131), seed=660 + G + T)
    t = wl.generate(w)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pq = oracle.quant_int8(oracle.prune(t.k, t.layout, a32, t.cu, T))
    mu, sigma = oracle.row_stats(t.k, t.layout, a32, t.cu)
    desc = make_desc(w, "HND")
    desc.stats = 1
    desc.pack_dtype = spark.PACK_INT8
    dk, dv, dq = to_dev(t.k), to_dev(t.v), to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(max(spark.packed_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    spark.prune(desc, dk, to_dev(t.qwin), dcu, packed)
    assert spark.check_packed(desc, packed) == 0
    mask = torch.empty((w.total, Hkv, 4), dtype=torch.int32, device="cuda")
    codes = torch.empty((w.total, Hkv, T), dtype=torch.int8, device="cuda")
    mup = torch.empty((w.total, Hkv), dtype=torch.float32, device="cuda")
    scale, mua, sg = torch.empty_like(mup), torch.empty_like(mup), torch.empty_like(mup)
    spark.unpack(desc, packed, mask, codes, mup, scale, None)
    spark.unpack_stats(desc, packed, mua, sg)
    torch.cuda.synchronize()
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), pq.mask)
    assert np.array_equal(codes.cpu().numpy(), pq.codes)
    assert np.array_equal(scale.cpu().numpy(), pq.scale)
    assert np.allclose(mup.cpu().numpy(), pq.mu32, rtol=1e-5, atol=1e-30)
    assert np.allclose(mua.cpu().numpy(), mu, rtol=1e-5, atol=1e-30)
    assert np.allclose(sg.cpu().numpy(), sigma, rtol=1e-5, atol=1e-6 * np.abs(mu).max())
    ws = spark.new_decode_workspace(desc)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    seed = 0xABCDEF0123456789 + T
    spark.decode_attn_sampled(desc, dq, packed, dv, dcu, out, ws, kind, seed)
    ref = oracle.decode_sampled(kind, seed, t.q, pq, mu, sigma, t.v, t.layout, t.cu)
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    print(f"{w.name}: max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS and np.all(out.cpu().numpy()[1] == 0)
    # the same cache under the degenerate recovery function
    spark.decode_attn(desc, dq, packed, dv, dcu, out, ws)
    ref0 = oracle.decode_literal(t.q, pq, t.v, t.layout, t.cu)
    assert np.abs(out.cpu().numpy().astype(np.float64) - ref0).max() <= MAX_ABS
