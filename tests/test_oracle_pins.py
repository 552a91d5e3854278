"""Pins for the CPU oracle: things the paper and the mathematics fix, none of which
is the oracle's own formula typed again.

* hand-worked cases (tests/golden/handworked.json), every intermediate value;
* keep-all (T = D) decode == dense attention, Eq. (4) == torch's softmax attention;
* brute force over all channel subsets: the kept set maximises Eq. (7), and among the
  maximisers it is the one preferring lower channel indices;
* exact-recovery construction: if every pruned entry already equals mu/a the method is
  lossless for any T, so the output equals dense attention;
* window-scale invariance, token-permutation invariance, convexity of the output,
  probabilities summing to one, order relations between kept / pruned saliencies;
* closed-form properties of the int8 storage variant.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
bf = wl.f32_to_bf16_bits
fb = wl.bf16_bits_to_f32


def _bits(x):
    x = np.asarray(x, dtype=np.float32)
    b = bf(x)
    assert np.array_equal(fb(b), x), "fixture value not representable in bfloat16"
    return b


def _kept_channels(mask_row, D):
    return [j for j in range(D) if (int(mask_row[j // 32]) >> (j % 32)) & 1]


# ------------------------------------------------------------------ hand-worked cases

with open(os.path.join(HERE, "golden", "handworked.json")) as fh:
    _CASES = json.load(fh)["cases"]


@pytest.mark.parametrize("case", _CASES, ids=[c["name"] for c in _CASES])
def test_handworked(case):
    B, Hq, Hkv, D, T, S = (case[x] for x in ("B", "Hq", "Hkv", "D", "T", "S"))
    qwin, k, v, q = _bits(case["qwin"]), _bits(case["k"]), _bits(case["v"]), _bits(case["q"])
    cu = np.array([0, S], np.int32)
    exp = case["expect"]

    qbar, a64, a32 = oracle.window_stat(qwin, Hkv)
    assert np.array_equal(a64, np.asarray(exp["a"], np.float64))
    assert np.array_equal(a32, np.asarray(exp["a"], np.float32))

    pr = oracle.prune(k, "NHD", a32, cu, T, want_w=True)
    assert np.array_equal(pr.w, np.asarray(exp["w"], np.float32))
    for n in range(S):
        for h in range(Hkv):
            assert _kept_channels(pr.mask[n, h], D) == exp["kept_channels"][n][h]
            want_vals = [case["k"][n][h][j] for j in exp["kept_channels"][n][h]]
            assert np.array_equal(fb(pr.kept[n, h]), np.asarray(want_vals, np.float32))
    assert np.array_equal(pr.mu64, np.asarray(exp["mu"], np.float64))
    assert np.array_equal(pr.mu32, np.asarray(exp["mu"], np.float32))

    out, probs = oracle.decode_literal(q, pr, v, "NHD", cu, want_probs=True)
    s = np.asarray(exp["scores"], np.float64)[0]          # [Hq, S]
    vv = np.asarray(case["v"], np.float64)                # [S, Hkv, D]
    G = Hq // Hkv
    for g in range(Hq):
        p0 = 1.0 / (1.0 + math.exp(s[g, 1] - s[g, 0]))     # logistic closed form for S = 2
        want_p = np.array([p0, 1.0 - p0])
        assert np.allclose(probs[g], want_p, rtol=0, atol=1e-15)
        want_o = want_p[0] * vv[0, g // G] + want_p[1] * vv[1, g // G]
        assert np.allclose(out[0, g], want_o, rtol=0, atol=1e-15)
    assert np.allclose(oracle.decode_fused(q, pr, v, "NHD", cu), out, rtol=0, atol=1e-14)


# ------------------------------------------------------------------ dense attention pins

def _random_small(seed, B=2, Hq=8, Hkv=2, D=128, W=8, seqlens=(37, 91), T=26, **kw):
    w = wl.small(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=D, window=W, keep=T,
                 seqlens=seqlens, seed=seed, **kw)
    return w, wl.generate(w)


def test_dense_attention_matches_library_softmax_attention():
    w, t = _random_small(1)
    out = oracle.dense_attn(t.q, t.k, t.v, t.layout, t.cu)
    G = w.n_q_heads // w.n_kv_heads
    kf = torch.from_numpy(fb(t.k).astype(np.float64))     # [Hkv, total, D]
    vf = torch.from_numpy(fb(t.v).astype(np.float64))
    qf = torch.from_numpy(fb(t.q).astype(np.float64))     # [B, Hq, D]
    for b in range(w.batch):
        s0, s1 = int(t.cu[b]), int(t.cu[b + 1])
        kk = kf[:, s0:s1].repeat_interleave(G, dim=0)[None]           # [1, Hq, S, D]
        vv = vf[:, s0:s1].repeat_interleave(G, dim=0)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(qf[b][None, :, None, :], kk, vv)
        assert np.allclose(out[b], ref[0, :, 0].numpy(), rtol=0, atol=1e-13)


@pytest.mark.parametrize("layout", ["HND", "NHD"])
def test_keep_all_is_dense_attention(layout):
    w, t = _random_small(2, T=128)
    k, v = t.k, t.v
    if layout == "NHD":
        k = np.ascontiguousarray(k.transpose(1, 0, 2))
        v = np.ascontiguousarray(v.transpose(1, 0, 2))
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(k, layout, a32, t.cu, 128)
    assert np.all(pr.mask == 0xFFFFFFFF) and np.all(pr.mu32 == 0) and np.all(np.isinf(pr.gap))
    kept_ref = k if layout == "NHD" else k.transpose(1, 0, 2)
    assert np.array_equal(pr.kept, kept_ref)
    dense = oracle.dense_attn(t.q, k, v, layout, t.cu)
    assert np.allclose(oracle.decode_literal(t.q, pr, v, layout, t.cu), dense, rtol=0, atol=1e-14)
    assert np.allclose(oracle.decode_fused(t.q, pr, v, layout, t.cu), dense, rtol=0, atol=1e-13)


# ------------------------------------------------------------------ selection pins

@pytest.mark.parametrize("D,T", [(6, 1), (7, 3), (8, 4), (9, 2), (10, 5), (10, 9)])
def test_selection_is_the_brute_force_optimum(D, T):
    rng = np.random.default_rng(100 + 10 * D + T)
    S, Hkv = 40, 2
    # few distinct magnitudes so ties (also across the cut) are common
    k = rng.integers(-3, 4, size=(S, Hkv, D)).astype(np.float32) * 0.5
    a32 = rng.integers(0, 3, size=(1, Hkv, D)).astype(np.float32) * 0.5   # zeros included
    cu = np.array([0, S], np.int32)
    pr = oracle.prune(bf(k), "NHD", a32, cu, T, want_w=True)
    for n in range(S):
        for h in range(Hkv):
            wrow = (a32[0, h].astype(np.float64) * np.abs(k[n, h]).astype(np.float64))
            assert np.array_equal(pr.w[n, h].astype(np.float64), wrow)    # products exact here
            best, best_sets = -1.0, []
            for sub in itertools.combinations(range(D), T):
                tot = float(sum(wrow[j] for j in sub))
                if tot > best + 1e-12:
                    best, best_sets = tot, [sub]
                elif abs(tot - best) <= 1e-12:
                    best_sets.append(sub)
            got = tuple(_kept_channels(pr.mask[n, h], D))
            assert len(got) == T
            assert got in best_sets                       # attains the maximum of Eq. (7)
            assert got == min(best_sets)                  # ties resolved towards lower channels
            pruned = [j for j in range(D) if j not in got]
            assert pr.mu64[n, h] == pytest.approx(np.mean(wrow[pruned]), abs=1e-15)


def test_selection_invariants_and_gqa_sharing():
    w, t = _random_small(3, Hq=8, Hkv=2, T=26)
    qbar, a64, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    # independent statement of the group weight: mean over the group's heads of |window mean|
    qf = fb(t.qwin).astype(np.float64)                                   # [B,Hq,W,D]
    G = w.n_q_heads // w.n_kv_heads
    a_ref = np.abs(qf.mean(axis=2)).reshape(w.batch, w.n_kv_heads, G, w.head_dim).mean(axis=2)
    assert np.allclose(a64, a_ref, rtol=0, atol=1e-15)
    assert np.array_equal(a32, a_ref.astype(np.float32)) or np.allclose(a32, a_ref, rtol=1e-7)

    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep, want_w=True)
    D, T = w.head_dim, w.keep
    bits = np.unpackbits(pr.mask.view(np.uint8), axis=-1, bitorder="little").astype(bool)   # [total,Hkv,D]
    assert np.all(bits.sum(-1) == T)                                       # exactly T per (token, head)
    wk = np.where(bits, pr.w, np.inf).min(-1)
    wp = np.where(~bits, pr.w, -np.inf).max(-1)
    assert np.all(wk >= wp)                                                # kept >= pruned
    assert np.all(pr.mu64 <= wk + 1e-15) and np.all(pr.mu64 >= 0)
    # on equality across the cut, every kept tied channel precedes every pruned tied channel
    for n, h in zip(*np.nonzero(wk == wp)):
        tied = np.nonzero(pr.w[n, h] == wk[n, h])[0]
        kept_t = [j for j in tied if bits[n, h, j]]
        prun_t = [j for j in tied if not bits[n, h, j]]
        assert max(kept_t) < min(prun_t)
    # K-hat holds the original bits of the kept channels, ascending
    kk = t.k.transpose(1, 0, 2)
    for n in (0, 5, w.total - 1):
        for h in range(w.n_kv_heads):
            assert np.array_equal(pr.kept[n, h], kk[n, h][bits[n, h]])
    # recovery consistency: a_j * ktilde_tj == mu_t for pruned entries (checked through the
    # literal decode in test_exact_recovery...); here: gap is the margin at the cut
    srt = -np.sort(-pr.w.astype(np.float64), axis=-1)
    assert np.allclose(pr.gap, (srt[..., T - 1] - srt[..., T]) / srt[..., T - 1], rtol=0, atol=1e-15)


def test_ties_and_zero_rows_keep_lowest_channels():
    D, T = 128, 26
    k = np.zeros((3, 1, D), np.float32)
    k[1] = 1.0                       # every saliency equal
    k[2, 0, 100:] = 2.0              # 28 large equal values, 26 kept -> channels 100..125
    a32 = np.ones((1, 1, D), np.float32)
    pr = oracle.prune(bf(k), "NHD", a32, np.array([0, 3], np.int32), T)
    assert _kept_channels(pr.mask[0, 0], D) == list(range(26))
    assert _kept_channels(pr.mask[1, 0], D) == list(range(26))
    assert _kept_channels(pr.mask[2, 0], D) == list(range(100, 126))
    assert pr.near_ties() == 3


# ------------------------------------------------------------------ recovery pins

def test_exact_recovery_construction_equals_dense_attention():
    """If every pruned entry already equals +mu/a, K-tilde == K and SparK is lossless."""
    rng = np.random.default_rng(7)
    B, Hq, Hkv, D, S = 2, 4, 2, 128, 50
    G = Hq // Hkv
    # window of one query whose entries are +-2^e  => a is a power of two per channel
    e = rng.integers(-2, 3, size=(B, Hkv, D))
    sign = rng.choice([-1.0, 1.0], size=(B, Hq, 1, D))
    qwin = sign * np.exp2(np.repeat(e, G, axis=1))[:, :, None, :]
    cu = np.array([0, S, 2 * S], np.int32)
    for T in (1, 26, 64, 127):
        k = np.empty((2 * S, Hkv, D), np.float32)
        for n in range(2 * S):
            b = n // S
            for h in range(Hkv):
                a = np.exp2(e[b, h])
                m = np.exp2(rng.integers(-6, -2))                    # the row's pruned saliency
                keep = rng.choice(D, size=T, replace=False)
                row = m / a                                          # pruned entries: + mu / a
                big = rng.choice([-1.0, 1.0], size=T) * rng.integers(2, 9, size=T) * m / a[keep]
                row[keep] = big                                      # kept: saliency >= 2m
                k[n, h] = row
        kb, vb = _bits(k), bf(rng.standard_normal((2 * S, Hkv, D)).astype(np.float32))
        qb = bf(rng.standard_normal((B, Hq, D)).astype(np.float32))
        _, _, a32 = oracle.window_stat(_bits(qwin), Hkv)
        assert np.array_equal(a32, np.exp2(e).astype(np.float32))
        pr = oracle.prune(kb, "NHD", a32, cu, T)
        dense = oracle.dense_attn(qb, kb, vb, "NHD", cu)
        assert np.allclose(oracle.decode_literal(qb, pr, vb, "NHD", cu), dense, rtol=0, atol=1e-13)
        assert np.allclose(oracle.decode_fused(qb, pr, vb, "NHD", cu), dense, rtol=0, atol=1e-11)


def test_recovered_entries_are_nonnegative_mu_over_a():
    """Lossy case: flipping the sign of a pruned key entry cannot change the output
    (the method stores no sign), while flipping a kept entry must."""
    w, t = _random_small(4, T=26)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    base = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    bits = np.unpackbits(pr.mask.view(np.uint8), axis=-1, bitorder="little").astype(bool)
    k2 = t.k.copy()
    flip = ~bits.transpose(1, 0, 2)                    # pruned entries, [Hkv,total,D]
    k2[flip] ^= np.uint16(0x8000)
    pr2 = oracle.prune(k2, t.layout, a32, t.cu, w.keep)
    assert np.array_equal(pr2.mask, pr.mask)
    assert np.array_equal(oracle.decode_literal(t.q, pr2, t.v, t.layout, t.cu), base)
    k3 = t.k.copy()
    k3[~flip] ^= np.uint16(0x8000)
    pr3 = oracle.prune(k3, t.layout, a32, t.cu, w.keep)
    assert np.array_equal(pr3.mask, pr.mask)
    assert np.abs(oracle.decode_literal(t.q, pr3, t.v, t.layout, t.cu) - base).max() > 1e-3


def test_zero_weight_channel_recovers_to_zero():
    w, t = _random_small(5, Hq=2, Hkv=2, T=26)
    qw = t.qwin.copy()
    qw[:, :, :, 3] = 0            # channel 3: window mean 0 -> a = 0 -> saliency 0 -> always pruned
    _, _, a32 = oracle.window_stat(qw, w.n_kv_heads)
    assert np.all(a32[:, :, 3] == 0)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    assert not np.any(pr.mask[..., 0] & np.uint32(8))
    out = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    assert np.all(np.isfinite(out))
    q2 = t.q.copy()
    q2[:, :, 3] = bf(np.float32(1000.0))      # the decode query's channel 3 meets a recovered 0
    assert np.allclose(oracle.decode_literal(q2, pr, t.v, t.layout, t.cu), out, rtol=0, atol=1e-13)
    assert np.allclose(oracle.decode_fused(t.q, pr, t.v, t.layout, t.cu), out, rtol=0, atol=1e-11)


def test_window_scale_invariance():
    w, t = _random_small(6, T=38)
    _, _, a1 = oracle.window_stat(t.qwin, w.n_kv_heads)
    qw4 = bf(fb(t.qwin) * np.float32(4.0))
    _, _, a4 = oracle.window_stat(qw4, w.n_kv_heads)
    p1 = oracle.prune(t.k, t.layout, a1, t.cu, w.keep)
    p4 = oracle.prune(t.k, t.layout, a4, t.cu, w.keep)
    assert np.array_equal(p1.mask, p4.mask) and np.array_equal(p4.mu32, 4 * p1.mu32)
    o1 = oracle.decode_literal(t.q, p1, t.v, t.layout, t.cu)
    o4 = oracle.decode_literal(t.q, p4, t.v, t.layout, t.cu)
    assert np.array_equal(o1, o4)


# ------------------------------------------------------------------ softmax / PV pins

def test_softmax_rows_and_convexity_and_permutation():
    w, t = _random_small(8, B=1, seqlens=(120,), T=26)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    out, probs = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu, want_probs=True)
    assert np.allclose(probs.sum(-1), 1.0, rtol=0, atol=1e-14) and np.all(probs >= 0)
    vf = fb(t.v).astype(np.float64)
    G = w.n_q_heads // w.n_kv_heads
    for g in range(w.n_q_heads):
        assert np.all(out[0, g] <= vf[g // G].max(0) + 1e-14)
        assert np.all(out[0, g] >= vf[g // G].min(0) - 1e-14)
    perm = np.random.default_rng(0).permutation(w.total)
    k2, v2 = np.ascontiguousarray(t.k[:, perm]), np.ascontiguousarray(t.v[:, perm])
    pr2 = oracle.prune(k2, t.layout, a32, t.cu, w.keep)
    assert np.array_equal(pr2.mask, pr.mask[perm])
    out2 = oracle.decode_literal(t.q, pr2, v2, t.layout, t.cu)
    assert np.allclose(out2, out, rtol=0, atol=1e-13)


def test_literal_and_fused_forms_agree_and_ragged_batches_are_independent():
    w, t = _random_small(9, B=3, seqlens=(64, 1, 130), T=25)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    lit = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    fus = oracle.decode_fused(t.q, pr, t.v, t.layout, t.cu)
    assert np.abs(lit - fus).max() < 1e-11
    # a sequence of length 1 attends to its only token: output is that V row exactly
    vf = fb(t.v).astype(np.float64)
    G = w.n_q_heads // w.n_kv_heads
    for g in range(w.n_q_heads):
        assert np.array_equal(lit[1, g], vf[g // G, 64])
    # running one sequence alone gives the same rows
    sl = slice(65, 195)
    _, _, a_b = oracle.window_stat(t.qwin[2:3], w.n_kv_heads)
    pr_b = oracle.prune(np.ascontiguousarray(t.k[:, sl]), "HND", a_b, np.array([0, 130], np.int32), 25)
    alone = oracle.decode_literal(t.q[2:3], pr_b, np.ascontiguousarray(t.v[:, sl]), "HND",
                                  np.array([0, 130], np.int32))
    assert np.array_equal(alone[0], lit[2])


def test_empty_sequence_gives_zero_output():
    w, t = _random_small(10, B=2, seqlens=(0, 33), T=26)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    out = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    assert np.all(out[0] == 0) and np.all(np.isfinite(out[1])) and np.any(out[1] != 0)


# ------------------------------------------------------------------ int8 storage variant

def test_int8_variant_closed_form_properties():
    w, t = _random_small(12, T=26)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    pq = oracle.quant_int8(pr)
    kf = fb(pr.kept).astype(np.float64)
    amax = np.abs(kf).max(-1)
    assert np.array_equal(pq.scale, (amax.astype(np.float32) / np.float32(127)).astype(np.float32))
    imax = np.abs(kf).argmax(-1)
    cmax = np.take_along_axis(pq.codes, imax[..., None], -1)[..., 0]
    assert np.all(np.abs(cmax.astype(int)) == 127)
    deq = pq.codes.astype(np.float64) * pq.scale.astype(np.float64)[..., None]
    # half a step, plus the binary32 rounding of the quotient (|k/scale| <= 127, eps = 2^-24)
    assert np.all(np.abs(deq - kf) <= pq.scale[..., None] * (0.5 + 127 * 2.0 ** -23))
    assert np.all(np.sign(pq.codes) * np.sign(kf) >= 0)
    # score perturbation bound: |ds| <= scale/2 * sum_kept |q_j| / sqrt(D); outputs stay close
    # hence every probability moves by at most a factor exp(+-2 * max_t |ds|)
    o_b, p_b = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu, want_probs=True)
    o_q, p_q = oracle.decode_literal(t.q, pq, t.v, t.layout, t.cu, want_probs=True)
    assert np.abs(o_b - o_q).max() > 0
    G = w.n_q_heads // w.n_kv_heads
    qabs = np.abs(fb(t.q).astype(np.float64)).sum(-1) / math.sqrt(w.head_dim)     # [B,Hq]
    for b in range(w.batch):
        sl = slice(int(t.cu[b]), int(t.cu[b + 1]))
        for g in range(w.n_q_heads):
            ds = (0.5 + 127 * 2.0 ** -23) * pq.scale[sl, g // G].astype(np.float64).max() * qabs[b, g]
            ratio = p_q[g, sl] / p_b[g, sl]
            assert np.all(ratio <= math.exp(2 * ds) * (1 + 1e-12))
            assert np.all(ratio >= math.exp(-2 * ds) * (1 - 1e-12))
    zero = oracle.Pruned(pr.mask[:1], np.zeros_like(pr.kept[:1]), pr.mu64[:1], pr.mu32[:1],
                         pr.gap[:1], pr.a32, None, pr.T, pr.D)
    zq = oracle.quant_int8(zero)
    assert np.all(zq.scale == 0) and np.all(zq.codes == 0)


# ------------------------------------------------------------------ value-cache pruning pins

with open(os.path.join(HERE, "golden", "handworked.json")) as fh:
    _VCASES = json.load(fh)["value_cases"]


@pytest.mark.parametrize("case", _VCASES, ids=[c["name"] for c in _VCASES])
def test_handworked_value_pruning(case):
    kc = next(c for c in _CASES if c["name"] == case["key_case"])
    Hkv, D, T, S = (kc[x] for x in ("Hkv", "D", "T", "S"))
    qwin, k, q, v = _bits(kc["qwin"]), _bits(kc["k"]), _bits(kc["q"]), _bits(case["v"])
    cu = np.array([0, S], np.int32)
    exp = case["expect"]
    _, _, a32 = oracle.window_stat(qwin, Hkv)
    pr = oracle.prune(k, "NHD", a32, cu, T)
    pv = oracle.prune_values(v, "NHD", case["Tv"])
    for n in range(S):
        assert _kept_channels(pv.mask[n, 0], D) == exp["kept_channels"][n][0]
    assert np.array_equal(fb(pv.kept), np.asarray(exp["kept_values"], np.float32))
    vt = oracle.expand_values(pv)
    assert np.array_equal(fb(vt), np.asarray(exp["vtilde"], np.float32))
    out = oracle.decode_literal(q, pr, vt, "NHD", cu)
    assert np.allclose(out, np.asarray(exp["out"], np.float64), rtol=0, atol=1e-15)


@pytest.mark.parametrize("D,Tv", [(6, 1), (7, 3), (8, 4), (10, 5), (10, 9)])
def test_value_selection_is_the_brute_force_optimum(D, Tv):
    """The kept set maximises the retained magnitude sum over all C(D, Tv) subsets, and among the
    maximisers it is the lexicographically smallest (ties towards lower channels)."""
    rng = np.random.default_rng(300 + 10 * D + Tv)
    S, Hkv = 40, 2
    v = rng.integers(-3, 4, size=(S, Hkv, D)).astype(np.float32) * 0.5     # many ties, zeros
    pv = oracle.prune_values(bf(v), "NHD", Tv)
    for n in range(S):
        for h in range(Hkv):
            mag = np.abs(v[n, h]).astype(np.float64)
            best, best_sets = -1.0, []
            for sub in itertools.combinations(range(D), Tv):
                tot = float(sum(mag[j] for j in sub))
                if tot > best + 1e-12:
                    best, best_sets = tot, [sub]
                elif abs(tot - best) <= 1e-12:
                    best_sets.append(sub)
            got = tuple(_kept_channels(pv.mask[n, h], D))
            assert len(got) == Tv and got in best_sets and got == min(best_sets)
            assert np.array_equal(fb(pv.kept[n, h]), v[n, h][list(got)])


def test_value_pruning_invariants_layouts_and_masked_product():
    w, t = _random_small(11, Hq=8, Hkv=2, T=26)
    D, Tv = w.head_dim, 48
    vf = fb(t.v)                                                          # [Hkv,total,D]
    pv = oracle.prune_values(t.v, t.layout, Tv)
    pv2 = oracle.prune_values(np.ascontiguousarray(t.v.transpose(1, 0, 2)), "NHD", Tv)
    assert np.array_equal(pv.mask, pv2.mask) and np.array_equal(pv.kept, pv2.kept)   # layout-independent
    bits = np.unpackbits(pv.mask.view(np.uint8), axis=-1, bitorder="little").astype(bool)   # [total,Hkv,D]
    assert np.all(bits.sum(-1) == Tv)
    mag = np.abs(vf).transpose(1, 0, 2)                                   # [total,Hkv,D]
    kept_min = np.where(bits, mag, np.inf).min(-1)
    pruned_max = np.where(~bits, mag, -np.inf).max(-1)
    assert np.all(kept_min >= pruned_max)
    # on equality across the cut the kept channel has the lower index
    for n, h in zip(*np.nonzero(kept_min == pruned_max)):
        c = kept_min[n, h]
        kept_eq = [j for j in range(D) if bits[n, h, j] and mag[n, h, j] == c]
        pruned_eq = [j for j in range(D) if not bits[n, h, j] and mag[n, h, j] == c]
        assert max(kept_eq) < min(pruned_eq)
    # the expanded rows are the original rows times the 0/1 mask, and decode over them is the
    # probability-weighted sum of those masked rows (probabilities do not depend on V)
    vt = oracle.expand_values(pv)
    assert np.array_equal(fb(vt), np.where(bits, vf.transpose(1, 0, 2), 0.0).astype(np.float32))
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    out, probs = oracle.decode_literal(t.q, pr, vt, "NHD", t.cu, want_probs=True)
    _, probs_dense_v = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu, want_probs=True)
    assert np.array_equal(probs, probs_dense_v)
    G = w.n_q_heads // w.n_kv_heads
    masked = np.where(bits, vf.transpose(1, 0, 2), 0.0).astype(np.float64)
    for b in range(w.batch):
        n0, n1 = int(t.cu[b]), int(t.cu[b + 1])
        for g in range(w.n_q_heads):
            ref = probs[g, n0:n1] @ masked[n0:n1, g // G, :]
            assert np.allclose(out[b, g], ref, rtol=0, atol=1e-13)


def test_keep_all_values_is_the_unpruned_value_cache():
    w, t = _random_small(12, Hq=4, Hkv=2, T=26)
    pv = oracle.prune_values(t.v, t.layout, w.head_dim)
    assert np.all(np.isinf(pv.gap))
    vt = oracle.expand_values(pv)
    assert np.array_equal(vt, t.v.transpose(1, 0, 2))


# ------------------------------------------------------------------ appended (never pruned) tokens

with open(os.path.join(HERE, "golden", "handworked.json")) as fh:
    _TCASES = json.load(fh)["tail_cases"]


@pytest.mark.parametrize("case", _TCASES, ids=[c["name"] for c in _TCASES])
def test_handworked_tail(case):
    kc = next(c for c in _CASES if c["name"] == case["key_case"])
    Hkv, T, S = (kc[x] for x in ("Hkv", "T", "S"))
    qwin, k, v, q = _bits(kc["qwin"]), _bits(kc["k"]), _bits(kc["v"]), _bits(kc["q"])
    cu = np.array([0, S], np.int32)
    _, _, a32 = oracle.window_stat(qwin, Hkv)
    pr = oracle.prune(k, "NHD", a32, cu, T)
    out = oracle.decode_literal_tail(q, pr, v, "NHD", cu, _bits(case["tail_k"]), _bits(case["tail_v"]),
                                     np.asarray(case["tail_len"], np.int32))
    assert np.allclose(out, np.asarray(case["expect"]["out"], np.float64), rtol=0, atol=1e-15)


def _random_tail(w, seed, cap):
    rng = np.random.default_rng(seed)
    shape = (w.batch, cap, w.n_kv_heads, w.head_dim)
    tk = bf(rng.standard_normal(shape).astype(np.float32))
    tv = bf(rng.standard_normal(shape).astype(np.float32))
    tl = rng.integers(0, cap + 1, size=w.batch).astype(np.int32)
    return tk, tv, tl


def test_tail_keep_all_is_dense_attention_on_the_concatenated_cache():
    w, t = _random_small(21, Hq=8, Hkv=2, T=128)
    tk, tv, tl = _random_tail(w, 21, cap=9)
    tl[:] = (9, 4)                                                        # full buffer, partly filled buffer
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.head_dim)               # T = D: nothing pruned
    got = oracle.decode_literal_tail(t.q, pr, t.v, t.layout, t.cu, tk, tv, tl)
    # the same cache written out as one dense cache per sequence: prefix rows, then appended rows
    kk = t.k.transpose(1, 0, 2)                                           # [total,Hkv,D]
    vv = t.v.transpose(1, 0, 2)
    ks, vs, cu2 = [], [], [0]
    for b in range(w.batch):
        n0, n1 = int(t.cu[b]), int(t.cu[b + 1])
        ks += [kk[n0:n1], tk[b, :tl[b]]]
        vs += [vv[n0:n1], tv[b, :tl[b]]]
        cu2.append(cu2[-1] + (n1 - n0) + int(tl[b]))
    ref = oracle.dense_attn(t.q, np.ascontiguousarray(np.concatenate(ks)), np.ascontiguousarray(np.concatenate(vs)),
                            "NHD", np.asarray(cu2, np.int32))
    assert np.allclose(got, ref, rtol=0, atol=1e-13)


def test_tail_empty_is_plain_decode_and_tail_only_is_dense_attention():
    w, t = _random_small(22, Hq=4, Hkv=2, T=26)
    tk, tv, tl = _random_tail(w, 22, cap=5)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    zero = np.zeros(w.batch, np.int32)
    assert np.array_equal(oracle.decode_literal_tail(t.q, pr, t.v, t.layout, t.cu, tk, tv, zero),
                          oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu))
    # a sequence with no prefix: attention over its appended rows alone
    w0, t0 = _random_small(23, Hq=4, Hkv=2, T=26)
    cu0 = np.zeros(w0.batch + 1, np.int32)
    empty = oracle.prune(t0.k[:, :0], t0.layout, a32[:w0.batch], cu0, w0.keep)
    tl2 = np.full(w0.batch, 5, np.int32)
    got = oracle.decode_literal_tail(t0.q, empty, t0.v[:, :0], t0.layout, cu0, tk[:w0.batch], tv[:w0.batch], tl2)
    cu5 = (np.arange(w0.batch + 1) * 5).astype(np.int32)
    ref = oracle.dense_attn(t0.q, np.ascontiguousarray(tk[:w0.batch].reshape(-1, w0.n_kv_heads, w0.head_dim)),
                            np.ascontiguousarray(tv[:w0.batch].reshape(-1, w0.n_kv_heads, w0.head_dim)), "NHD", cu5)
    assert np.allclose(got, ref, rtol=0, atol=1e-13)


# ------------------------------------------------------------------ sampled recovery pins

def _unmix32(y):
    """Inverse of the 32-bit mixer, derived independently: undo each xor-shift, multiply by the modular
    inverse of each odd constant."""
    M = 0xFFFFFFFF
    y ^= y >> 16
    y = (y * pow(0xC2B2AE35, -1, 1 << 32)) & M
    y ^= (y >> 13) ^ (y >> 26)
    y = (y * pow(0x85EBCA6B, -1, 1 << 32)) & M
    y ^= y >> 16
    return y


def test_generator_is_a_bijective_mixer_and_its_uniforms_behave():
    rng = np.random.default_rng(31)
    for x in [0, 1, 2, 0xFFFFFFFF] + [int(v) for v in rng.integers(0, 1 << 32, size=200)]:
        assert _unmix32(oracle.mix32(x)) == x
    assert oracle.mix32(0) == 0
    # uniforms: in (0,1), on the 23-bit grid offset by half a step, deterministic, sensitive to every argument
    u = np.array([[oracle.uniform(1234567890123, n, 1, c) for c in range(128)] for n in range(400)])
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.all((u * (1 << 23) - 0.5) == np.round(u * (1 << 23) - 0.5))
    assert oracle.uniform(7, 3, 1, 5) == oracle.uniform(7, 3, 1, 5)
    base = oracle.uniform(7, 3, 1, 5)
    assert len({base, oracle.uniform(8, 3, 1, 5), oracle.uniform(7 + (1 << 32), 3, 1, 5), oracle.uniform(7, 4, 1, 5),
                oracle.uniform(7, 3, 2, 5), oracle.uniform(7, 3, 1, 6)}) == 6
    flat = u.reshape(-1)                                       # 51,200 draws
    assert abs(flat.mean() - 0.5) < 0.005 and abs(flat.var() - 1.0 / 12.0) < 0.002
    assert abs(np.corrcoef(u[:, :-1].reshape(-1), u[:, 1:].reshape(-1))[0, 1]) < 0.02     # neighbouring counters
    assert abs(np.corrcoef(u[:-1].reshape(-1), u[1:].reshape(-1))[0, 1]) < 0.02           # neighbouring tokens
    hist = np.histogram(flat, bins=16, range=(0, 1))[0]
    assert hist.min() > 0.9 * flat.size / 16 and hist.max() < 1.1 * flat.size / 16


def _header_generator_text():
    with open(os.path.join(os.path.dirname(HERE), "include", "spark.h")) as fh:
        return fh.read()


def _uniform_from_the_header(seed, n, h, c):
    """The generator exactly as include/spark.h words it, in Python integers (no oracle call):
    mix(x): x ^= x >> 16; x *= 0x85EBCA6B; x ^= x >> 13; x *= 0xC2B2AE35; x ^= x >> 16 on 32-bit words,
    base = mix(mix(mix(n) + seed_lo) + h * 0x9E3779B9 + seed_hi), x_c = mix(base + c * 0x9E3779B9),
    u_c = ((x_c >> 9) + 0.5) / 2^23.  Returns (x_c, u_c as an exact fraction numerator over 2^24)."""
    M = 0xFFFFFFFF

    def mix(x):
        x &= M
        x ^= x >> 16
        x = (x * 0x85EBCA6B) & M
        x ^= x >> 13
        x = (x * 0xC2B2AE35) & M
        x ^= x >> 16
        return x

    seed_lo, seed_hi = seed & M, (seed >> 32) & M
    base = mix((mix((mix(n) + seed_lo) & M) + h * 0x9E3779B9 + seed_hi) & M)
    x = mix((base + c * 0x9E3779B9) & M)
    return x, 2 * (x >> 9) + 1          # u = (2 * (x >> 9) + 1) / 2^24


def test_generator_known_answers_from_the_header_text():
    """Holds the oracle's uniforms to the generator written out in include/spark.h: the composition (which
    word is added where, the stride of the counter, the order of the three mixes) is recomputed here with
    Python integers for a spread of arguments and must agree exactly, bit for bit."""
    text = _header_generator_text()
    for token in ("0x85EBCA6B", "0xC2B2AE35", "0x9E3779B9", "x >> 16", "x >> 13", "(x_c >> 9) + 0.5"):
        assert token in text, f"the header no longer states {token}"
    # the mixer alone, two values computed by hand from the five steps (x = 1 and x = 0xFFFFFFFF)
    assert oracle.mix32(1) == 0x514E28B7 and oracle.mix32(0xFFFFFFFF) == 0x81F16F39
    rng = np.random.default_rng(77)
    cases = [(0, 0, 0, 0), (1, 0, 0, 0), (0, 1, 0, 0), (0, 0, 1, 0), (0, 0, 0, 1), (1 << 32, 0, 0, 0),
             (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF, 7, 127), (0x5EED0002, 2097151, 7, 101)]
    cases += [(int(rng.integers(0, 1 << 63)), int(rng.integers(0, 1 << 31)), int(rng.integers(0, 64)),
               int(rng.integers(0, 128))) for _ in range(300)]
    for seed, n, h, c in cases:
        x, num = _uniform_from_the_header(seed, n, h, c)
        u = oracle.uniform(seed, n, h, c)
        assert u * (1 << 24) == num, (seed, n, h, c, x)
    # neighbouring counters, heads and tokens are separated by the stated strides, not by some other constant
    x0, _ = _uniform_from_the_header(123, 5, 1, 0)
    x1, _ = _uniform_from_the_header(123, 5, 1, 1)
    assert x0 != x1 and _unmix32(x1) == (_unmix32(x0) + 0x9E3779B9) & 0xFFFFFFFF


def _sampled_setup(seed, T=26):
    w, t = _random_small(seed, Hq=8, Hkv=2, T=T)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep, want_w=True)
    mu, sigma = oracle.row_stats(t.k, t.layout, a32, t.cu)
    return w, t, a32, pr, mu, sigma


def test_row_statistics_are_mean_and_population_std_of_the_saliency():
    w, t, a32, pr, mu, sigma = _sampled_setup(41)
    wf = pr.w.astype(np.float64)                               # [total,Hkv,D], the compared products
    assert np.allclose(mu, wf.mean(-1), rtol=1e-7, atol=0)
    assert np.allclose(sigma, wf.std(-1), rtol=1e-6, atol=0)   # numpy's std is the population one
    # the mean of the pruned set lies below the all-channel mean (the largest entries were kept)
    assert np.all(pr.mu64 <= mu.astype(np.float64) * (1 + 1e-6))


@pytest.mark.parametrize("kind", [oracle.GAUSSIAN, oracle.EXPONENTIAL])
def test_sampled_decode_is_plain_attention_over_the_exported_rebuilt_keys(kind):
    w, t, a32, pr, mu, sigma = _sampled_setup(42)
    out, kt = oracle.decode_sampled(kind, 99, t.q, pr, mu, sigma, t.v, t.layout, t.cu, want_ktilde=True)
    bits = np.unpackbits(pr.mask.view(np.uint8), axis=-1, bitorder="little").astype(bool)
    kf = fb(t.k).transpose(1, 0, 2).astype(np.float64)         # [total,Hkv,D]
    assert np.array_equal(kt[bits], kf[bits])                  # kept entries are the original ones
    qf, vf = fb(t.q).astype(np.float64), fb(t.v).transpose(1, 0, 2).astype(np.float64)
    G = w.n_q_heads // w.n_kv_heads
    for b in range(w.batch):
        n0, n1 = int(t.cu[b]), int(t.cu[b + 1])
        for g in range(w.n_q_heads):
            s = kt[n0:n1, g // G, :] @ qf[b, g] / math.sqrt(w.head_dim)
            p = np.exp(s - s.max())
            p /= p.sum()
            assert np.allclose(out[b, g], p @ vf[n0:n1, g // G, :], rtol=0, atol=1e-12)
    # another seed gives other pruned entries, the same kept ones
    _, kt2 = oracle.decode_sampled(kind, 100, t.q, pr, mu, sigma, t.v, t.layout, t.cu, want_ktilde=True)
    assert np.array_equal(kt2[bits], kt[bits]) and not np.array_equal(kt2[~bits], kt[~bits])


@pytest.mark.parametrize("kind", [oracle.GAUSSIAN, oracle.EXPONENTIAL])
def test_sampled_decode_over_int8_kept_entries(kind):
    """The int8 storage variant under a sampled recovery function: kept entries are code * scale (the codes and
    scales of the degenerate path, computed after selection), pruned entries are the very samples of the bf16
    run (the statistics are those of the saliencies before quantisation), and the output is plain attention
    over those rebuilt keys."""
    w, t, a32, pr, mu, sigma = _sampled_setup(43)
    pq = oracle.quant_int8(pr)
    out, kt = oracle.decode_sampled(kind, 77, t.q, pq, mu, sigma, t.v, t.layout, t.cu, want_ktilde=True)
    _, kt_bf16 = oracle.decode_sampled(kind, 77, t.q, pr, mu, sigma, t.v, t.layout, t.cu, want_ktilde=True)
    bits = np.unpackbits(pr.mask.view(np.uint8), axis=-1, bitorder="little").astype(bool)
    deq = pq.codes.astype(np.float64) * pq.scale.astype(np.float64)[..., None]      # [total,Hkv,T], channel order
    assert np.array_equal(kt[bits], deq.reshape(-1))
    assert np.array_equal(kt[~bits], kt_bf16[~bits])
    assert np.abs(kt[bits] - kt_bf16[bits]).max() <= 0.5 * pq.scale.max() * (1 + 1e-6)   # half a quantisation step
    qf, vf = fb(t.q).astype(np.float64), fb(t.v).transpose(1, 0, 2).astype(np.float64)
    G = w.n_q_heads // w.n_kv_heads
    for b in range(w.batch):
        n0, n1 = int(t.cu[b]), int(t.cu[b + 1])
        for g in range(w.n_q_heads):
            s = kt[n0:n1, g // G, :] @ qf[b, g] / math.sqrt(w.head_dim)
            p = np.exp(s - s.max())
            p /= p.sum()
            assert np.allclose(out[b, g], p @ vf[n0:n1, g // G, :], rtol=0, atol=1e-12)


@pytest.mark.parametrize("kind", [oracle.GAUSSIAN, oracle.EXPONENTIAL])
def test_sampled_entries_have_the_moments_of_their_distribution(kind):
    """Rebuilt pruned entries times a are the sampled saliencies: Gaussian N(mu, sigma^2), Exponential with
    mean mu (hence standard deviation mu), per row; checked through standardised samples over many rows."""
    w, t, a32, pr, mu, sigma = _sampled_setup(43)
    _, kt = oracle.decode_sampled(kind, 7, t.q, pr, mu, sigma, t.v, t.layout, t.cu, want_ktilde=True)
    bits = np.unpackbits(pr.mask.view(np.uint8), axis=-1, bitorder="little").astype(bool)
    cu = np.asarray(t.cu)
    seq = np.searchsorted(cu, np.arange(w.total), side="right") - 1
    a_rows = a32[seq].astype(np.float64)                       # [total,Hkv,D]
    wt = kt * a_rows                                           # sampled saliency where pruned and a != 0
    sel = (~bits) & (a_rows != 0)
    m, sd = mu.astype(np.float64)[..., None], sigma.astype(np.float64)[..., None]
    if kind == oracle.GAUSSIAN:
        z = ((wt - m) / sd)[sel]
        assert abs(z.mean()) < 0.02 and abs(z.std() - 1.0) < 0.02
        assert abs(((z ** 3).mean())) < 0.05 and abs((z ** 4).mean() - 3.0) < 0.15
        assert (wt[sel] < 0).any()                             # not clamped
    else:
        e = (wt / m)[sel]
        assert e.min() > 0 and abs(e.mean() - 1.0) < 0.02 and abs(e.std() - 1.0) < 0.03
        assert abs(np.mean(e > math.log(2.0)) - 0.5) < 0.01    # median of the unit exponential


def test_gaussian_recovery_with_zero_spread_is_the_degenerate_recovery_at_the_row_mean():
    """Rows whose saliencies are all equal have sigma = 0 and mu = mu_pruned, so the Gaussian recovery
    function returns mu for every pruned entry: exactly the degenerate function."""
    w, t = _random_small(44, Hq=4, Hkv=2, T=26)
    rng = np.random.default_rng(44)
    t.k = bf(rng.choice([-2.0, 2.0], size=t.k.shape).astype(np.float32))     # |k| constant
    t.qwin = bf(np.ones(t.qwin.shape, np.float32))                           # a constant (= 1)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune(t.k, t.layout, a32, t.cu, w.keep)
    mu, sigma = oracle.row_stats(t.k, t.layout, a32, t.cu)
    assert np.all(sigma == 0) and np.array_equal(mu, pr.mu32)
    got = oracle.decode_sampled(oracle.GAUSSIAN, 5, t.q, pr, mu, sigma, t.v, t.layout, t.cu)
    assert np.allclose(got, oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu), rtol=0, atol=1e-14)


def test_gaussian_pairs_are_the_box_muller_transform_of_their_two_uniforms():
    """Channels 2m, 2m+1 share one radius and one angle: z0^2 + z1^2 = -2 ln u_(2m) and the angle of
    (z0, z1) is 2 pi u_(2m+1); so the two samples of a pair are uncorrelated, not copies."""
    w, t, a32, pr, mu, sigma = _sampled_setup(45)
    seed = 0xABCDEF0123
    _, kt = oracle.decode_sampled(oracle.GAUSSIAN, seed, t.q, pr, mu, sigma, t.v, t.layout, t.cu, want_ktilde=True)
    bits = np.unpackbits(pr.mask.view(np.uint8), axis=-1, bitorder="little").astype(bool)
    cu = np.asarray(t.cu)
    checked = 0
    z0s, z1s = [], []
    for n in range(0, w.total, 7):
        b = int(np.searchsorted(cu, n, side="right") - 1)
        for h in range(w.n_kv_heads):
            for m in range(64):
                j = 2 * m
                if bits[n, h, j] or bits[n, h, j + 1] or a32[b, h, j] == 0 or a32[b, h, j + 1] == 0:
                    continue
                z0 = (kt[n, h, j] * float(a32[b, h, j]) - float(mu[n, h])) / float(sigma[n, h])
                z1 = (kt[n, h, j + 1] * float(a32[b, h, j + 1]) - float(mu[n, h])) / float(sigma[n, h])
                u1, u2 = oracle.uniform(seed, n, h, j), oracle.uniform(seed, n, h, j + 1)
                assert z0 * z0 + z1 * z1 == pytest.approx(-2.0 * math.log(u1), rel=1e-9)
                ang = math.atan2(z1, z0) % (2 * math.pi)
                assert min(abs(ang - 2 * math.pi * u2), 2 * math.pi - abs(ang - 2 * math.pi * u2)) < 1e-7
                z0s.append(z0)
                z1s.append(z1)
                checked += 1
    assert checked > 500
    assert abs(np.corrcoef(z0s, z1s)[0, 1]) < 0.1


# ------------------------------------------------------------------ top-p variant pins

def _topp_rows(k_rows, a_row, p_bp=9900):
    """Runs the oracle's top-p pruning on hand-made rows: k_rows [S, D] floats (bf16-exact), a_row [D] floats that
    are exact as the mean |window query| of a one-query window.  Returns the Pruned and the float32 saliencies."""
    k_rows = np.asarray(k_rows, np.float32)
    S, D = k_rows.shape
    qwin = _bits(np.asarray(a_row, np.float32).reshape(1, 1, 1, D))
    _, _, a32 = oracle.window_stat(qwin, 1)
    assert np.array_equal(a32.reshape(-1), np.asarray(a_row, np.float32))
    k = _bits(k_rows.reshape(S, 1, D))
    pr = oracle.prune_topp(k, "NHD", a32, np.array([0, S], np.int32), p_bp)
    w = (a32.reshape(1, D) * np.abs(k_rows)).astype(np.float32)      # one float32 multiply per entry
    return pr, w


def test_topp_count_is_the_shortest_prefix_by_exact_rational_arithmetic():
    """Brute force over every prefix length of tiny rows, in exact fractions of the float32 saliencies (not the
    oracle's integer units): the kept count is the first m whose m largest saliencies reach 99 % of the total,
    no shorter prefix does, and the kept set is the m largest with ties to the lower channel."""
    from fractions import Fraction
    rng = np.random.default_rng(91)
    checked = 0
    for D in (3, 5, 8, 10):
        for trial in range(40):
            a_row = _q(rng.uniform(0.25, 4.0, size=D))
            k_rows = _q(rng.standard_normal((6, D)) * rng.choice([1.0, 8.0, 0.01], size=(1, D)))
            pr, w = _topp_rows(k_rows, a_row)
            for t in range(k_rows.shape[0]):
                ws = [Fraction(float(x)) for x in w[t]]
                order = sorted(range(D), key=lambda j: (-ws[j], j))
                tot = sum(ws)
                cum, m = Fraction(0), 0
                margins = []
                while True:
                    cum += ws[order[m]]
                    m += 1
                    margins.append(abs(cum - Fraction(99, 100) * tot))
                    if cum >= Fraction(99, 100) * tot or m == D:
                        break
                if tot > 0 and min(margins) < Fraction(1, 10**5) * tot:
                    continue          # (a prefix sum within 1e-5 of the cut: the integer units may decide either way)
                assert int(pr.count[t, 0]) == m, (D, trial, t)
                assert _kept_channels(pr.mask[t, 0], D) == sorted(order[:m])
                assert np.array_equal(fb(pr.kept[t, 0, :m]), k_rows[t, sorted(order[:m])])
                assert np.all(pr.kept[t, 0, m:] == 0)
                pruned = [ws[j] for j in order[m:]]
                want_mu = float(sum(pruned) / len(pruned)) if pruned else 0.0
                assert pr.mu64[t, 0] == pytest.approx(want_mu, rel=1e-12, abs=0)
                checked += 1
    assert checked > 600


def _q(x):
    """Round to bfloat16-representable float32 values."""
    return fb(bf(np.asarray(x, np.float32)))


def test_topp_special_rows():
    D = 128
    ones = np.ones(D, np.float32)
    # one dominant channel: 99.5 % of the total sits in channel 17 -> one channel kept
    k = np.full((1, D), 1.0, np.float32)
    k[0, 17] = 32768.0            # 32768 / (32768 + 127) = 0.9961
    pr, _ = _topp_rows(k, ones)
    assert pr.count[0, 0] == 1 and _kept_channels(pr.mask[0, 0], D) == [17]
    # ... just below 99 %: the dominant one plus as many equal small ones (lowest channels) as it takes
    k[0, 17] = 8192.0             # 8192 / 8319 = 0.9847;  (8192 + n) >= 0.99 * 8319 = 8235.81  ->  n = 44
    pr, _ = _topp_rows(k, ones)
    assert pr.count[0, 0] == 45
    assert _kept_channels(pr.mask[0, 0], D) == sorted([17] + list(range(0, 17)) + list(range(18, 45)))
    # equal saliencies: ceil(0.99 * 128) = 127 channels, the lowest ones
    pr, _ = _topp_rows(np.full((1, D), 3.0, np.float32), ones)
    assert pr.count[0, 0] == 127 and _kept_channels(pr.mask[0, 0], D) == list(range(127))
    assert pr.mu64[0, 0] == 3.0
    # p = 100 %: every channel with a saliency that counts; zero channels are dropped, and mu is then 0
    k = np.zeros((1, D), np.float32)
    k[0, 5:50] = np.linspace(1, 2, 45, dtype=np.float32)
    pr, _ = _topp_rows(_q(k), ones, p_bp=10000)
    assert pr.count[0, 0] == 45 and _kept_channels(pr.mask[0, 0], D) == list(range(5, 50))
    assert pr.mu64[0, 0] == 0.0
    # the unit is the last place of the row's largest saliency, no coarser: three saliencies of exactly one unit
    # (2^-23 beside 1.0) count at p = 100 % (total 2^23 + 3 units: all four channels are needed), and at 99.99 %
    # the largest alone is enough (need = ceil(0.9999 * (2^23 + 3)) <= 2^23)
    k = np.zeros((1, D), np.float32)
    k[0, 40] = 1.0
    k[0, [3, 77, 101]] = 2.0 ** -23
    pr, _ = _topp_rows(k, ones, p_bp=10000)
    assert pr.count[0, 0] == 4 and _kept_channels(pr.mask[0, 0], D) == [3, 40, 77, 101]
    pr, _ = _topp_rows(k, ones, p_bp=9999)
    assert pr.count[0, 0] == 1 and _kept_channels(pr.mask[0, 0], D) == [40]
    # ... and no finer: half a unit is rounded down to nothing (2^-24 beside 1.0 never counts)
    k[0, [3, 77, 101]] = 2.0 ** -24
    pr, _ = _topp_rows(k, ones, p_bp=10000)
    assert pr.count[0, 0] == 1 and _kept_channels(pr.mask[0, 0], D) == [40]
    # an all-zero row keeps exactly one channel, the first
    pr, _ = _topp_rows(np.zeros((2, D), np.float32), ones)
    assert np.all(pr.count == 1) and _kept_channels(pr.mask[1, 0], D) == [0]
    # a smaller p keeps fewer: counts are monotone in p
    rng = np.random.default_rng(92)
    k = _q(rng.standard_normal((20, D)))
    a = _q(rng.uniform(0.5, 2.0, size=D))
    counts = [_topp_rows(k, a, p_bp)[0].count[:, 0] for p_bp in (5000, 9000, 9900, 9990, 10000)]
    for lo, hi in zip(counts[:-1], counts[1:]):
        assert np.all(lo <= hi)
    assert np.all(counts[-1] == D) or np.any(np.abs(k) == 0)


def test_topp_prefix_property_and_decode_on_random_data():
    """On benchmark-like rows: the kept saliencies reach 99 % of the total and would not without the smallest kept
    one (float64 sums, with a margin for the integer units); the kept set is a top set; decode over the rebuilt
    keys is the literal recovery followed by Eq. (4), and a row that keeps everything reproduces dense attention."""
    w, t = _random_small(61, Hq=8, Hkv=2, T=26)
    _, _, a32 = oracle.window_stat(t.qwin, w.n_kv_heads)
    pr = oracle.prune_topp(t.k, t.layout, a32, t.cu, 9900)
    full = oracle.prune(t.k, t.layout, a32, t.cu, w.head_dim, want_w=True)      # (for the saliencies w)
    wf = full.w.astype(np.float64)
    bits = np.unpackbits(pr.mask.view(np.uint8), axis=-1, bitorder="little").astype(bool)
    assert np.array_equal(bits.sum(-1), pr.count)
    tot = wf.sum(-1)
    kept_sum = (wf * bits).sum(-1)
    smallest_kept = np.where(bits, wf, np.inf).min(-1)
    largest_pruned = np.where(~bits, wf, -np.inf).max(-1)
    assert np.all(kept_sum >= 0.99 * tot * (1 - 1e-5))
    assert np.all((kept_sum - smallest_kept < 0.99 * tot * (1 + 1e-5)) | (pr.count == 1))
    assert np.all(smallest_kept >= largest_pruned)
    # the same count selected with the fixed-count rule gives the same set (the top-p set is a top-T set)
    for n in range(0, w.total, 17):
        for h in range(w.n_kv_heads):
            T_row = int(pr.count[n, h])
            one = oracle.prune(np.ascontiguousarray(t.k[:, n:n + 1]), t.layout, a32[:1] if n < t.cu[1] else a32[1:2],
                               np.array([0, 1], np.int32), T_row)
            assert np.array_equal(one.mask[0, h], pr.mask[n, h])
            assert one.mu64[0, h] == pr.mu64[n, h]
    # decode: literal form == factored form; at p = 100 % (every row keeps all non-zero channels) == dense attention
    out = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
    assert np.allclose(oracle.decode_fused(t.q, pr, t.v, t.layout, t.cu), out, rtol=0, atol=1e-12)
    allp = oracle.prune_topp(t.k, t.layout, a32, t.cu, 10000)
    if np.all(allp.count == w.head_dim):
        assert np.allclose(oracle.decode_literal(t.q, allp, t.v, t.layout, t.cu),
                           oracle.dense_attn(t.q, t.k, t.v, t.layout, t.cu), rtol=0, atol=1e-13)
