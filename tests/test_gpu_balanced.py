"""GPU parity for the balanced cut of decode: the (sequence, tile) items of a KV head dealt out in equal
contiguous ranges to independent wavefronts, one partial per (wavefront, sequence), merged by whoever counts in
last.  The library picks it for batches of 32 to 256 short sequences; `n_splits = -1` asks for it on any batch,
which is how the small cases here reach it.  Same oracle and tolerance as plain decode."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import make_desc, to_dev
from tests.test_gpu_parity import _run
from tests.test_gpu_tail import _tail_case

pytestmark = pytest.mark.gpu


def test_ragged_with_empty_and_single_token_sequences():
    res, _, _ = _run(wl.small(name="bal_edges", batch=6, seqlens=(0, 1, 63, 64, 65, 0), keep=26, seed=60), n_splits=-1)
    assert np.all(res["out_f32"][0] == 0) and np.all(res["out_f32"][5] == 0)


@pytest.mark.parametrize("G,Hkv", [(1, 2), (2, 2), (4, 2), (8, 2), (16, 1)])
def test_group_sizes(G, Hkv):
    # (16 query heads per KV head have no balanced form: the request falls back to the cut by length)
    _run(wl.small(name=f"bal_gqa{G}", n_q_heads=G * Hkv, n_kv_heads=Hkv, keep=26, seqlens=(257, 64, 190), batch=3,
                  seed=600 + G), n_splits=-1)


@pytest.mark.parametrize("T", [1, 25, 26, 27, 38, 64, 128])
def test_keep_values(T):
    _run(wl.small(name=f"bal_keep{T}", keep=T, seqlens=(130, 321), seed=620 + T), n_splits=-1)


def test_int8_storage():
    _run(wl.small(name="bal_int8", keep=26, seqlens=(300, 141), seed=640), int8=True, n_splits=-1)
    _run(wl.small(name="bal_int8_t25", keep=25, seqlens=(100, 70, 0, 33), batch=4, seed=641), int8=True, n_splits=-1)
    _run(wl.small(name="bal_int8_t64", keep=64, seqlens=(300, 141, 77), batch=3, seed=642), int8=True, n_splits=-1)


def test_token_major_layout():
    _run(wl.small(name="bal_nhd", seqlens=(333, 129), seed=645), layout="NHD", n_splits=-1)


def test_one_long_sequence_among_short_ones_gets_many_partials():
    """Fewer items than wavefronts: every item is a wavefront's whole range, the long sequence ends up with 141
    partials (nine merge rounds of sixteen), the empty one with the single spare partial id."""
    _run(wl.small(name="bal_skewed", batch=7, n_q_heads=8, n_kv_heads=2, keep=26,
                  seqlens=(9000, 64, 0, 700, 1, 130, 2500), seed=650), n_splits=-1)


def test_ranges_that_span_several_sequences():
    """Many KV heads leave 64 wavefronts per head: with some 200 items a head, a wavefront's range holds three or
    four tiles and crosses sequence boundaries (store a partial, rebuild the table, go on), including runs of
    empty sequences and sequences that share a tile with their neighbours."""
    rng = np.random.default_rng(660)
    lens = [int(x) for x in rng.integers(0, 600, size=40)]
    lens[3] = lens[4] = lens[5] = 0
    lens[10], lens[11], lens[12] = 5, 1, 7
    w = wl.small(name="bal_spans", batch=40, n_q_heads=32, n_kv_heads=32, keep=26, seqlens=tuple(lens), seed=660)
    _run(w)          # 40 * 32 pairs: the library chooses the balanced cut by itself
    _run(w, n_splits=-1, want_unpack=True)


def test_batch_of_empty_sequences_gives_zero_output():
    w = wl.small(name="bal_allempty", batch=2, n_q_heads=4, n_kv_heads=2, keep=26, seqlens=(0, 0), seed=1)
    t = wl.generate(w)
    desc = make_desc(w, n_splits=-1)
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


def test_appended_rows_are_counted_in_with_the_wavefronts_partials():
    w = wl.small(name="bal_tail", batch=6, seqlens=(0, 1, 63, 300, 65, 0), keep=26, seed=670)
    got, _ = _tail_case(w, cap=300, tail_len=(5, 0, 300, 1, 0, 0), seed=670, n_splits=-1)
    assert np.all(got[5] == 0)


def test_repeated_calls_on_one_workspace_leave_the_counters_clear():
    """The arrival counters wrap to zero at the last arrival, also when wavefronts (not blocks) count in: the
    same workspace serves the balanced and the length-proportional cut in turn, bit for bit each time."""
    w = wl.small(name="bal_repeat", batch=5, n_q_heads=8, n_kv_heads=2, keep=26, seqlens=(700, 64, 0, 1300, 190), seed=680)
    t = wl.generate(w)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    ref = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    d_bal, d_len = make_desc(w, n_splits=-1), make_desc(w)
    dk, dv, dqw, dq = to_dev(t.k), to_dev(t.v), to_dev(t.qwin), to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(max(spark.packed_bytes(d_bal), 256), dtype=torch.uint8, device="cuda")
    spark.prune(d_bal, dk, dqw, dcu, packed)
    assert spark.decode_workspace_bytes(d_bal) >= spark.decode_workspace_bytes(d_len)
    ws = spark.new_decode_workspace(d_bal)
    first = {}
    for it in range(6):
        d = d_bal if it % 2 == 0 else d_len
        out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
        spark.decode_attn(d, dq, packed, dv, dcu, out, ws)
        got = out.cpu().numpy()
        assert np.abs(got - ref).max() <= 1e-2
        if it % 2 not in first:
            first[it % 2] = got
        assert np.array_equal(got, first[it % 2])


def test_both_cuts_agree_on_larger_random_batches():
    """Sizes the oracle would take minutes for: forty seeded batches of 1 to 256 sequences - random, log-uniform,
    equal, equal with holes, mostly empty - head counts, row lengths and storage varied, a quarter of them with
    appended rows; the balanced cut (asked for, and the library's own choice) against one block per sequence on
    the same cache, each call made twice on its workspace.  The cuts differ in summation order only."""
    rng = np.random.default_rng(7001)
    for case in range(40):
        hkv = int(rng.choice([1, 2, 4, 8, 16, 32]))
        G = int(rng.choice([1, 2, 4, 8]))
        B = int(rng.integers(1, 257)) if rng.random() < 0.7 else int(rng.choice([32, 64, 128, 256]))
        T = int(rng.choice([26, 64, 38, 25, int(rng.integers(1, 129))]))
        kind = int(rng.integers(0, 5))
        top = int(rng.choice([100, 600, 2500]))
        if kind == 0:
            lens = rng.integers(0, top, size=B)
        elif kind == 1:
            lens = np.exp(rng.uniform(0, np.log(top), size=B)).astype(np.int64)
        elif kind == 2:
            lens = np.full(B, int(rng.choice([64, 128, 512, 192, 65])))
        elif kind == 3:
            lens = np.full(B, int(rng.choice([64, 256, 512])))
            lens[rng.integers(0, B, size=max(1, B // 8))] = 0
        else:
            lens = np.zeros(B, np.int64)
            lens[rng.integers(0, B, size=max(1, B // 6))] = rng.integers(1, top, size=max(1, B // 6))
        lens = [int(x) for x in lens]
        int8, tail = bool(rng.integers(0, 2)), rng.random() < 0.25
        if sum(lens) == 0 or sum(lens) * hkv > 2_000_000:
            continue
        w = wl.small(name=f"bal_rand{case}", batch=B, n_q_heads=G * hkv, n_kv_heads=hkv, keep=T, seqlens=tuple(lens),
                     seed=7100 + case)
        t = wl.generate(w)
        pack = spark.PACK_INT8 if int8 else spark.PACK_BF16
        cap = 40 if tail else 0
        descs = []
        for ns in (-1, 1, 0):
            d = make_desc(w, pack=pack, n_splits=ns)
            d.tail_capacity = cap
            descs.append(d)
        dk, dv, dqw, dq = to_dev(t.k), to_dev(t.v), to_dev(t.qwin), to_dev(t.q)
        dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
        packed = torch.empty(max(spark.packed_bytes(descs[0]), 256), dtype=torch.uint8, device="cuda")
        spark.prune(descs[0], dk, dqw, dcu, packed)
        if tail:
            shape = (B, cap, hkv, w.head_dim)
            tk = to_dev(wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32)))
            tv = to_dev(wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32)))
            tl = torch.from_numpy(rng.integers(0, cap + 1, size=B).astype(np.int32)).cuda()
        outs = []
        for d in descs:
            out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
            ws = spark.new_decode_workspace(d)
            for _ in range(2):
                if tail:
                    spark.decode_attn_tail(d, dq, packed, dv, dcu, tk, tv, tl, out, ws)
                else:
                    spark.decode_attn(d, dq, packed, dv, dcu, out, ws)
            outs.append(out.cpu().numpy())
        diff = max(np.abs(outs[0] - outs[1]).max(), np.abs(outs[2] - outs[1]).max())
        print(f"case {case}: B={B} Hkv={hkv} G={G} T={T} lengths {kind} int8={int8} tail={tail} tokens={sum(lens)} "
              f"max|diff|={diff:.2e}", flush=True)
        assert all(np.all(np.isfinite(o)) for o in outs) and diff <= 3e-4
        if not tail:
            for i, n in enumerate(lens):
                if n == 0:
                    assert np.all(outs[0][i] == 0) and np.all(outs[2][i] == 0)


def test_longest_sequence_hint_keeps_one_block_per_sequence_on_even_batches():
    """desc.max_seqlen within 9/8 of the average: the batch is balanced as it is and the library does not deal it
    out to wavefronts - same cut, so bit for bit the same result, as n_splits = 1; a hint that says "ragged", or
    none, leaves the balanced cut on."""
    rng = np.random.default_rng(690)
    lens = tuple(int(x) for x in rng.integers(780, 820, size=48))         # (600 tiles: two per wavefront and more)
    w = wl.small(name="bal_hint", batch=48, n_q_heads=32, n_kv_heads=8, keep=26, seqlens=lens, seed=690)
    t = wl.generate(w)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    ref = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    dk, dv, dqw, dq = to_dev(t.k), to_dev(t.v), to_dev(t.qwin), to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    outs = {}
    for tag, ns, hint in (("one", 1, 0), ("even", 0, max(lens)), ("ragged", 0, 4 * max(lens)), ("none", 0, 0)):
        d = make_desc(w, n_splits=ns)
        d.max_seqlen = hint
        packed = torch.empty(max(spark.packed_bytes(d), 256), dtype=torch.uint8, device="cuda")
        spark.prune(d, dk, dqw, dcu, packed)
        out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
        spark.decode_attn(d, dq, packed, dv, dcu, out, spark.new_decode_workspace(d))
        outs[tag] = out.cpu().numpy()
        assert np.abs(outs[tag] - ref).max() <= 1e-2
    assert np.array_equal(outs["even"], outs["one"])
    assert np.array_equal(outs["ragged"], outs["none"])
    assert not np.array_equal(outs["none"], outs["one"])        # (another summation order)


def test_sequences_that_are_exactly_one_blocks_share():
    """64 equal sequences x 8 KV heads, 256 wavefronts per head: every sequence is the share of one block's four
    wavefronts, whose states are folded through LDS and written out without partials in memory; then the same
    with one sequence cut short, so that most pairs still align with blocks and the ones after it do not."""
    w = wl.small(name="bal_aligned", batch=64, n_q_heads=32, n_kv_heads=8, keep=26, seqlens=(512,) * 64, seed=700)
    _run(w)
    # sequences without tokens are looked after by the wavefront of their number: here wavefronts of blocks whose
    # pair is folded through LDS (sequences 0 .. 4 still align with blocks 0 .. 4; wavefronts 5, 6, 7 sit in block 1)
    lens = [512] * 64
    lens[5] = lens[6] = lens[7] = 0
    _run(wl.small(name="bal_aligned_empty", batch=64, n_q_heads=32, n_kv_heads=8, keep=26, seqlens=tuple(lens), seed=702))
    lens = [512] * 64
    lens[20] = 130
    _run(wl.small(name="bal_misaligned", batch=64, n_q_heads=32, n_kv_heads=8, keep=64, seqlens=tuple(lens), seed=701))
