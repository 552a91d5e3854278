"""GPU parity for the top-p variant (per row, the fewest channels that hold p of the row's saliency): per-row
counts, masks and kept entries bit-exact against the CPU oracle (both sides decide the count in the same integer
arithmetic), mu to 1e-5 relative, decode output within the decode tolerance; small ragged shapes, the special
rows (one dominant channel, equal saliencies, zero rows, ties at the cut) and the 32K benchmark shape."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import make_desc, to_dev

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 1e-2, 1e-3


def _run(w, t, p_bp=9900, layout="HND", decode=True, n_splits=0):
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune_topp(t.k, t.layout, a32, t.cu, p_bp)
    k, v = t.k, t.v
    if layout == "NHD":
        k = np.ascontiguousarray(k.transpose(1, 0, 2))
        v = np.ascontiguousarray(v.transpose(1, 0, 2))
    desc = make_desc(w, layout, n_splits=n_splits)
    dk, dv, dq = to_dev(k), to_dev(v), to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.zeros(max(spark.packed_topp_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    spark.prune_topp(desc, dk, to_dev(t.qwin), dcu, p_bp, packed)
    total, hkv, D = w.total, w.n_kv_heads, w.head_dim
    mask = torch.empty((total, hkv, 4), dtype=torch.int32, device="cuda")
    count = torch.empty((total, hkv), dtype=torch.int32, device="cuda")
    vals = torch.empty((total, hkv, D), dtype=torch.int16, device="cuda")
    mu = torch.empty((total, hkv), dtype=torch.float32, device="cuda")
    a = torch.empty((w.batch, hkv, D), dtype=torch.float32, device="cuda")
    spark.unpack_topp(desc, packed, mask, count, vals, mu, a)
    torch.cuda.synchronize()
    cnt = count.cpu().numpy()
    print(f"{w.name}: rows={total * hkv} p={p_bp / 100:.2f}% kept per row: mean {cnt.mean():.1f} min {cnt.min()} max {cnt.max()}")
    assert np.array_equal(a.cpu().numpy(), a32)
    assert np.array_equal(cnt, pr.count), "per-row counts differ"
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), pr.mask), "kept-channel sets differ"
    assert np.array_equal(vals.cpu().numpy().view(np.uint16), pr.kept), "kept entries differ"
    assert np.allclose(mu.cpu().numpy(), pr.mu32, rtol=1e-5, atol=1e-30)
    if decode:
        out = torch.empty((w.batch, w.n_q_heads, D), dtype=torch.float32, device="cuda")
        spark.decode_attn_topp(desc, dq, packed, dv, dcu, out, spark.new_decode_workspace(desc))
        ref = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
        err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
        print(f"   decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
        assert np.all(np.isfinite(out.cpu().numpy()))
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS
    return pr


@pytest.mark.parametrize("p_bp", [9900, 9000, 5000, 10000, 1])
def test_small_ragged(p_bp):
    w = wl.small(name=f"topp{p_bp}", seqlens=(200, 77), seed=300 + p_bp % 97)
    _run(w, wl.generate(w), p_bp)


@pytest.mark.parametrize("G,Hkv", [(1, 2), (2, 2), (4, 2), (8, 1), (16, 1)])
def test_group_sizes(G, Hkv):
    w = wl.small(name=f"toppG{G}", n_q_heads=G * Hkv, n_kv_heads=Hkv, seqlens=(130, 321), seed=310 + G)
    _run(w, wl.generate(w))


def test_token_major_layout_and_split_counts():
    w = wl.small(name="toppNHD", seqlens=(700, 64, 1), seed=321, batch=3)
    t = wl.generate(w)
    _run(w, t, layout="NHD")
    for ns in (1, 3, 7):
        _run(w, t, n_splits=ns)


def test_empty_and_single_token_sequences():
    w = wl.small(name="toppempty", batch=5, seqlens=(0, 1, 130, 0, 64), seed=322)
    _run(w, wl.generate(w))


def test_special_rows():
    """One dominant channel, equal saliencies (ties at the cut: lowest channels win), zero rows, heavy outliers."""
    w = wl.small(name="toppspecial", batch=1, n_q_heads=4, n_kv_heads=1, seqlens=(192,), seed=323)
    t = wl.generate(w)
    k = wl.bf16_bits_to_f32(t.k).copy()            # [1, 192, 128]
    k[0, 0] = 1.0
    k[0, 0, 17] = 32768.0                          # dominant
    k[0, 1] = 3.0                                  # all equal (given equal channel weights below)
    k[0, 2] = 0.0                                  # zero row
    k[0, 3] = 0.0
    k[0, 3, 100] = -2.0                            # a single non-zero entry
    k[0, 4, :64] = 1.0                             # two plateaus: ties inside the cut
    k[0, 4, 64:] = 0.5
    k[0, 5] *= 1e-30                               # tiny row
    k[0, 6] *= 1e30                                # huge row
    k[0, 7] = 0.0                                  # saliencies of exactly one unit in the last place of the largest
    k[0, 7, 40] = 1.0
    k[0, 7, [3, 77, 101]] = 2.0 ** -23
    k[0, 8] = 0.0                                  # ... and of half a unit (rounded down to nothing)
    k[0, 8, 40] = 1.0
    k[0, 8, [3, 77, 101]] = 2.0 ** -24
    # one large key over a plateau of small ones that holds the cut: ten octaves down (far outside the window of
    # the selection's first level), in the window's last bin, and in the first bin outside it
    for row, small in ((9, 2.0 ** -10), (10, 1.125 * 2.0 ** -8), (11, 2.0 ** -8)):
        k[0, row] = small
        k[0, row, 5] = 1.0
    # ... and sixteen octaves down, where that window (four bins an octave) ends: its last bin and the first
    # outside it; the plateau holds the cut at p = 99.99 % and 100 %
    for row, small in ((12, 1.25 * 2.0 ** -16), (13, 2.0 ** -16), (14, 2.0 ** -20)):
        k[0, row] = small
        k[0, row, 77] = -1.0
    t.k = wl.f32_to_bf16_bits(k)
    t.qwin = wl.f32_to_bf16_bits(np.ones(t.qwin.shape, np.float32))      # a = 1 everywhere
    pr = _run(w, t)
    assert 100 < pr.count[9, 0] < 128 and 100 < pr.count[10, 0] < 128 and 100 < pr.count[11, 0] < 128
    assert pr.count[0, 0] == 1 and pr.count[1, 0] == 127 and pr.count[2, 0] == 1 and pr.count[3, 0] == 1
    pr = _run(w, t, p_bp=10000)
    assert pr.count[7, 0] == 4 and pr.count[8, 0] == 1
    pr = _run(w, t, p_bp=9999)
    assert 100 < pr.count[12, 0] < 128 and 100 < pr.count[13, 0] < 128 and pr.count[14, 0] < 128


def test_keys_concentrated_in_a_minority_of_channels():
    """The benchmark's recipe for this variant: 60 % of each head's key channels quiet, so that 99 % of a row's
    saliency sits in some fifty channels (the cut then falls between the loud and the quiet channels, seven
    octaves apart: near the end of the selection's first-level window)."""
    w = wl.small(name="toppquiet", batch=3, n_q_heads=16, n_kv_heads=4, seqlens=(700, 129, 300), seed=325)
    w.quiet_fraction, w.quiet_scale = 0.6, 0.008
    pr = _run(w, wl.generate(w))
    assert 35 < pr.count.mean() < 70
    _run(w, wl.generate(w), p_bp=9990)
    _run(w, wl.generate(w), p_bp=9000)


def test_config2_size():
    """The 32K benchmark shape (2.1 M rows): every count, mask and kept entry checked, decode checked."""
    w = wl.config(2)
    _run(w, wl.generate(w))
