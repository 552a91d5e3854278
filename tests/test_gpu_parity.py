"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Index work (masks, kept entries, channel weights, int8 codes) must match
bit for bit; floating point within the stated tolerance:

    decode output (float32 out):  max |err| <= 1e-2, mean |err| <= 1e-3   (bf16 in, fp32 accumulate)
    mu (float32 mean of <= 127 float32 saliencies, any summation order):  relative 1e-5

Near-ties (relative saliency gap < 1e-6 at the cut) are counted and printed; they are
expected to match as well because both sides compare the same float32 products.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import make_desc, run_gpu_case, to_dev

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3


def _oracle_all(w, t, int8=False):
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    if int8:
        pr = oracle.quant_int8(pr)
    ref = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    return a32, pr, ref


def _check_prune(res, a32, pr, int8=False):
    assert np.array_equal(res["a"], a32), "channel weights a differ"
    assert np.array_equal(res["mask"], pr.mask), "kept-channel sets differ"
    bits = np.unpackbits(res["mask"].view(np.uint8), axis=-1, bitorder="little")
    assert np.all(bits.sum(-1) == pr.T)
    if int8:
        assert np.array_equal(res["scale"], pr.scale)
        assert np.array_equal(res["vals"], pr.codes)
    else:
        assert np.array_equal(res["vals"], pr.kept), "kept entries differ"
    assert np.allclose(res["mu"], pr.mu32, rtol=1e-5, atol=1e-30)


def _check_out(res, ref, tag=""):
    err = np.abs(res["out_f32"].astype(np.float64) - ref)
    print(f"{tag} decode max|err|={err.max():.3e} mean|err|={err.mean():.3e}")
    assert np.all(np.isfinite(res["out_f32"]))
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS
    if "out_bf16" in res:
        # the bf16 output is the float32 output rounded to nearest even
        want = torch.from_numpy(res["out_f32"]).to(torch.bfloat16).float().numpy()
        assert np.array_equal(res["out_bf16"], want)


def _run(w, t=None, int8=False, **kw):
    t = wl.generate(w) if t is None else t
    a32, pr, ref = _oracle_all(w, t, int8)
    print(f"{w.name}: rows={w.total * w.n_kv_heads} near-ties(<1e-6)={pr.near_ties()}")
    res = run_gpu_case(w, t, pack=spark.PACK_INT8 if int8 else spark.PACK_BF16, **kw)
    _check_prune(res, a32, pr, int8)
    _check_out(res, ref, w.name)
    return res, pr, ref


def test_small_ragged_keep26():
    _run(wl.small())


def test_config1_tiny_1k_keep64():
    _run(wl.config(1))


@pytest.mark.parametrize("T", [1, 2, 25, 26, 27, 38, 64, 65, 127, 128])
def test_keep_values(T):
    # several tiles and a ragged tail; odd T exercises the half-filled last value word,
    # T = 128 is plain dense attention
    _run(wl.small(name=f"keep{T}", keep=T, seqlens=(130, 321), seed=20 + T))


@pytest.mark.parametrize("G,Hkv", [(1, 2), (2, 2), (4, 3), (8, 2), (16, 1)])
def test_group_sizes(G, Hkv):
    _run(wl.small(name=f"gqa{G}", n_q_heads=G * Hkv, n_kv_heads=Hkv, keep=26, seqlens=(257, 64, 190), batch=3,
                  seed=40 + G))


@pytest.mark.parametrize("layout", ["HND", "NHD"])
def test_layouts(layout):
    _run(wl.small(name=f"layout{layout}", seqlens=(333, 129), seed=50), layout=layout)


def test_ragged_with_empty_and_single_token_sequences():
    w = wl.small(name="ragged_edges", batch=6, seqlens=(0, 1, 63, 64, 65, 0), keep=26, seed=60)
    res, pr, ref = _run(w)
    assert np.all(res["out_f32"][0] == 0) and np.all(res["out_f32"][5] == 0)
    # one cached token: the output is that token's V row
    vf = wl.bf16_bits_to_f32(wl.generate(w).v)
    G = w.n_q_heads // w.n_kv_heads
    for g in range(w.n_q_heads):
        assert np.allclose(res["out_f32"][1, g], vf[g // G, 0], rtol=0, atol=1e-6)


@pytest.mark.parametrize("ns", [1, 2, 3, 7, 33])
def test_split_counts_agree(ns):
    w = wl.small(name=f"splits{ns}", batch=2, seqlens=(1500, 700), keep=26, seed=70)
    res, _, ref = _run(w, n_splits=ns)
    res1 = run_gpu_case(w, wl.generate(w), n_splits=1, want_unpack=False, want_bf16=False)
    assert np.abs(res["out_f32"] - res1["out_f32"]).max() < 1e-4


def test_constructed_ties_and_zero_rows():
    """Saliencies drawn from a handful of values: the cut falls inside a tie in most rows."""
    w = wl.small(name="ties", batch=2, n_q_heads=4, n_kv_heads=2, keep=26, seqlens=(150, 90), seed=80)
    t = wl.generate(w)
    rng = np.random.default_rng(80)
    kq = rng.integers(-2, 3, size=t.k.shape).astype(np.float32)
    kq[:, 10:20, :] = 0.0                          # all-zero rows: channels 0..T-1 kept
    kq[:, 30:40, :] = 1.0                          # all-equal rows
    t.k = wl.f32_to_bf16_bits(kq)
    t.qwin = wl.f32_to_bf16_bits(np.sign(wl.bf16_bits_to_f32(t.qwin)))   # |qbar| few distinct values
    a32, pr, ref = _oracle_all(w, t)
    assert pr.near_ties() > 0.5 * pr.gap.size
    res = run_gpu_case(w, t)
    _check_prune(res, a32, pr)
    _check_out(res, ref, "ties")


def test_int8_storage_variant():
    _run(wl.small(name="int8", keep=26, seqlens=(300, 141), seed=90), int8=True)
    _run(wl.small(name="int8_t25", keep=25, seqlens=(100, 70), seed=91), int8=True)
    # (row lengths with an instantiation of their own, and one without)
    _run(wl.small(name="int8_t38", keep=38, seqlens=(200, 131), seed=92), int8=True)
    _run(wl.small(name="int8_t64", keep=64, seqlens=(257, 64, 190), batch=3, n_q_heads=16, n_kv_heads=2, seed=93), int8=True)
    _run(wl.small(name="int8_t51", keep=51, seqlens=(150, 90), seed=94), int8=True)


def test_peaked_softmax_keeps_tolerance():
    """A decode query aligned with one key makes the softmax nearly one-hot; outlier V channels are
    large, so this is where a low-precision P would show."""
    w = wl.small(name="peaked", batch=1, n_q_heads=4, n_kv_heads=1, keep=64, seqlens=(700,), seed=95,
                 n_outlier=8, outlier_scale=10.0)
    t = wl.generate(w)
    kf = wl.bf16_bits_to_f32(t.k)
    q = np.stack([kf[0, 100] * 0.5, kf[0, 300] * 0.35, -kf[0, 5] * 0.3, kf[0, 650] * 0.2])[None]
    t.q = wl.f32_to_bf16_bits(q.astype(np.float32))
    _run(w, t)


def test_window_scale_invariance_on_gpu():
    w = wl.small(name="scale_inv", keep=38, seqlens=(200, 100), seed=97)
    t = wl.generate(w)
    r1 = run_gpu_case(w, t)
    t.qwin = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(t.qwin) * np.float32(4.0))
    r4 = run_gpu_case(w, t)
    assert np.array_equal(r1["mask"], r4["mask"])
    assert np.abs(r1["out_f32"] - r4["out_f32"]).max() < 1e-5


@pytest.mark.parametrize("lo,hi,with_decode", [(-12, 3, True), (-100, 20, False), (-145, -115, False)])
def test_token_scales_jump_by_many_octaves(lo, hi, with_decode):
    """Neighbouring tokens whose key norms differ by powers of two far apart: the threshold search
    starts each row from the previous row's exponent and has to walk up or down from it."""
    w = wl.small(name=f"octaves{lo}_{hi}", batch=2, n_q_heads=8, n_kv_heads=2, keep=26, seqlens=(200, 131), seed=99)
    t = wl.generate(w)
    rng = np.random.default_rng(99)
    kf = wl.bf16_bits_to_f32(t.k)                                   # [Hkv, total, D]
    e = rng.integers(lo, hi + 1, size=kf.shape[:2]).astype(np.float32)
    e[:, 5::17] = lo                                                # runs of abrupt changes
    e[:, 6::17] = hi
    t.k = wl.f32_to_bf16_bits((kf * np.exp2(e)[..., None]).astype(np.float32))   # exact: a power of two
    a32, pr, ref = _oracle_all(w, t)
    res = run_gpu_case(w, t)
    _check_prune(res, a32, pr)
    if with_decode:
        _check_out(res, ref, w.name)


def test_skewed_batch_long_sequences_get_more_blocks():
    """One long sequence among short ones: the library cuts sequences into blocks by length (the long one
    into many), short and empty ones get a single block."""
    w = wl.small(name="skewed", batch=7, n_q_heads=8, n_kv_heads=2, keep=26, seqlens=(9000, 64, 0, 700, 1, 130, 2500),
                 seed=120)
    res, _, _ = _run(w)
    assert np.all(res["out_f32"][2] == 0)


def test_batch_larger_than_the_chunk_numbering_handles_in_one_pass():
    """More than 256 sequences: every sequence gets the same number of blocks (the in-kernel numbering of
    length-proportional chunks works on 64 sequences at a time and is not used for very large batches)."""
    rng = np.random.default_rng(121)
    lens = tuple(int(x) for x in rng.integers(0, 90, size=300))
    w = wl.small(name="batch300", batch=300, n_q_heads=4, n_kv_heads=2, keep=26, seqlens=lens, seed=121)
    _run(w)


def test_batch_between_64_and_256_sequences():
    rng = np.random.default_rng(122)
    lens = tuple(int(x) for x in rng.integers(0, 200, size=150))
    w = wl.small(name="batch150", batch=150, n_q_heads=4, n_kv_heads=2, keep=26, seqlens=lens, seed=122)
    _run(w)


def test_batch_of_empty_sequences_gives_zero_output():
    """No cached token at all: prune launches nothing, decode still writes every output row (zeros)."""
    w = wl.small(name="allempty", batch=2, n_q_heads=4, n_kv_heads=2, keep=26, seqlens=(0, 0), seed=1)
    t = wl.generate(w)
    desc = make_desc(w)
    desc.k_head_stride = desc.v_head_stride = w.head_dim        # (zero tokens: any valid stride)
    dq = to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.zeros(max(spark.packed_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    k1 = torch.zeros(256, dtype=torch.int16, device="cuda")          # valid pointers; no row is ever read
    spark.prune(desc, k1, to_dev(t.qwin), dcu, packed)
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), 7.0, dtype=torch.float32, device="cuda")
    spark.decode_attn(desc, dq, packed, k1, dcu, out, spark.new_decode_workspace(desc))
    torch.cuda.synchronize()
    assert np.all(out.cpu().numpy() == 0)


def test_one_workspace_serves_descriptions_of_different_total_length():
    """The arrival counters sit at the start of the workspace, so a workspace prepared once serves batches of
    other total lengths (other block counts, other partial-state positions) with the same batch and KV heads."""
    ws_desc = make_desc(wl.small(name="wsbig", seqlens=(5000, 3000), seed=71))
    ws = torch.empty(2 * spark.decode_workspace_bytes(ws_desc), dtype=torch.uint8, device="cuda")
    ws.fill_(0xA5)                                   # garbage everywhere ...
    spark.decode_workspace_init(ws_desc, ws)         # ... except what the init call prepares
    for seqlens, seed in (((5000, 3000), 71), ((130, 77), 72), ((2500, 900), 73), ((64, 64), 74), ((5000, 3000), 71)):
        w = wl.small(name=f"ws{seqlens[0]}", seqlens=seqlens, seed=seed)
        t = wl.generate(w)
        a32, pr, ref = _oracle_all(w, t)
        res = run_gpu_case(w, t, want_unpack=False, want_bf16=False)      # fresh workspace: the reference run
        desc = res["desc"]
        assert spark.decode_workspace_bytes(desc) <= ws.numel()
        dk, dv, dqw, dq, dcu = res["dev"]
        out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        spark.decode_attn(desc, dq, res["packed"], dv, dcu, out, ws)
        got = out.cpu().numpy()
        assert np.array_equal(got, res["out_f32"]), seqlens
        err = np.abs(got.astype(np.float64) - ref)
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS


def test_check_packed_tells_matching_from_foreign_caches():
    w = wl.small(name="chk", seqlens=(200, 77), seed=75)
    t = wl.generate(w)
    res = run_gpu_case(w, t, want_unpack=False, want_bf16=False)
    desc, packed = res["desc"], res["packed"]
    assert spark.check_packed(desc, packed) == 0
    for field, val in (("keep", 27), ("pack_dtype", spark.PACK_INT8), ("stats", 1), ("total_tokens", w.total + 1),
                       ("n_kv_heads", 1), ("batch", 3)):
        d2 = spark.SparkDesc.from_buffer_copy(desc)
        setattr(d2, field, val)
        if field == "n_kv_heads":
            d2.n_q_heads = 4
        assert spark.check_packed(d2, packed) == spark.ERR_MISMATCH, field
    # a value cache is told apart from a key cache, and checked against keep_v
    dv_desc = spark.SparkDesc.from_buffer_copy(desc)
    dv_desc.keep_v = 64
    packed_v = torch.empty(spark.packed_values_bytes(dv_desc), dtype=torch.uint8, device="cuda")
    spark.prune_values(dv_desc, res["dev"][1], packed_v)
    assert spark.check_packed(dv_desc, packed_v, True) == 0
    assert spark.check_packed(dv_desc, packed_v, False) == spark.ERR_MISMATCH
    assert spark.check_packed(dv_desc, packed, True) == spark.ERR_MISMATCH
    dv_desc.keep_v = 38
    assert spark.check_packed(dv_desc, packed_v, True) == spark.ERR_MISMATCH


def test_non_finite_entries_stay_inside_their_sequence_and_head():
    """Inputs are expected to be finite; Inf / NaN entries are not detected.  The contract: the call completes, and
    rows, sequences and KV heads that hold no such entry are not affected."""
    w = wl.small(name="nonfinite", batch=4, n_q_heads=8, n_kv_heads=2, seqlens=(150, 260, 90, 200), seed=88)
    t = wl.generate(w)
    cu = np.asarray(t.cu)
    inf, nan = np.uint16(0x7F80), np.uint16(0x7FC1)
    # sequence 1, KV head 0: scattered Inf / -Inf / NaN key entries, one row full of NaN, one full of Inf
    for n, j, bits in ((cu[1] + 3, 5, inf), (cu[1] + 3, 77, np.uint16(0xFF80)), (cu[1] + 64, 0, nan), (cu[1] + 65, 127, nan)):
        t.k[0, n, j] = bits
    t.k[0, cu[1] + 100, :] = nan
    t.k[0, cu[1] + 101, :] = inf
    # sequence 3: a NaN and an Inf among the window queries of q head 5 (KV head 1)
    t.qwin[3, 5, 2, 10] = nan
    t.qwin[3, 5, 3, 11] = inf
    res = run_gpu_case(w, t, want_bf16=False)          # completes (every search loop is bounded)
    a32, pr, ref = _oracle_all(w, t)
    bad_rows = np.zeros((w.total, w.n_kv_heads), bool)
    bad_rows[cu[1]:cu[2], 0] = ~np.isfinite(wl.bf16_bits_to_f32(t.k[0, cu[1]:cu[2]])).all(-1)
    bad_rows[cu[3]:cu[4], 1] = True
    good = ~bad_rows
    assert np.array_equal(res["mask"][good], pr.mask[good]), "a clean row changed"
    assert np.array_equal(res["vals"][good], pr.kept[good])
    assert np.allclose(res["mu"][good], pr.mu32[good], rtol=1e-5, atol=1e-30)
    G = w.n_q_heads // w.n_kv_heads
    clean_out = np.ones((w.batch, w.n_q_heads), bool)
    clean_out[1, 0:G] = False             # q heads of KV head 0 in sequence 1
    clean_out[3, G:2 * G] = False         # q heads of KV head 1 in sequence 3
    err = np.abs(res["out_f32"].astype(np.float64) - ref)[clean_out]
    assert np.all(np.isfinite(res["out_f32"][clean_out]))
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS


def test_timeline_aid_changes_no_result_and_files_ordered_stamps():
    """The measurement aid of include/spark_bench.h: with a buffer given, every working block files five ordered
    wall-clock stamps and exactly one block per (batch, KV head) reports the merge; the output is bit for bit
    the one computed without it; a buffer too small for the grid files nothing."""
    w = wl.small(name="tline", seqlens=(5000, 3000, 0, 700), batch=4, seed=76)
    t = wl.generate(w)
    res = run_gpu_case(w, t, want_unpack=False, want_bf16=False)
    desc = res["desc"]
    dk, dv, dqw, dq, dcu = res["dev"]
    ws = spark.new_decode_workspace(desc)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    buf = torch.zeros(4096 * 8, dtype=torch.int64, device="cuda")
    spark.decode_timeline(buf)
    try:
        spark.decode_attn(desc, dq, res["packed"], dv, dcu, out, ws)
        torch.cuda.synchronize()
        tr = buf.cpu().numpy().reshape(-1, 8)
        small = torch.zeros(8, dtype=torch.int64, device="cuda")       # room for one block only
        spark.decode_timeline(small)
        spark.decode_attn(desc, dq, res["packed"], dv, dcu, out, ws)
        torch.cuda.synchronize()
        assert not small.cpu().numpy().any()
    finally:
        spark.decode_timeline(None)
    assert np.array_equal(out.cpu().numpy(), res["out_f32"])
    work = tr[(tr[:, 0] != 0) & (tr[:, 4] != 0)]
    assert len(work) >= w.batch * w.n_kv_heads
    assert np.all(work[:, 0] <= work[:, 1]) and np.all(work[:, 1] <= work[:, 2])
    assert np.all(work[:, 2] <= work[:, 3]) and np.all(work[:, 3] <= work[:, 4])
    assert (work[:, 4] - work[:, 0]).max() < 100 * 1000 * 100          # under 100 ms in 10 ns ticks
    tiles = sum((int(t.cu[i + 1]) - 1) // 64 - int(t.cu[i]) // 64 + 1 for i in range(w.batch) if t.cu[i + 1] > t.cu[i])
    assert work[:, 5].sum() == tiles * w.n_kv_heads
    # pairs cut into several blocks are merged by exactly one of them
    assert 0 < (work[:, 7] == 1).sum() <= w.batch * w.n_kv_heads


def test_profile_summaries_that_bench_reads_are_present_on_this_box():
    """bench.py takes roofline.traffic from a profile summary: the file has to travel with the tree."""
    import bench
    nbytes, src = bench.measured_traffic("cfg2_llama8b_b8_32k_keep26", "bf16")
    assert src == "profiles/decode_prune_cfg2_hbm_traffic.md" and nbytes and 0.9 < nbytes / 687865856 < 1.1
