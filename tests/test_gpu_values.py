"""GPU parity for value-cache channel pruning (the appendix extension that prunes keys and values
together): kept sets and kept entries bit for bit against the CPU oracle; decode over both packed
caches within the decode tolerance (max |err| <= 1e-2, mean |err| <= 1e-3)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import make_desc, to_dev

pytestmark = pytest.mark.gpu


def _prune_values_gpu(w, v_bits, Tv, layout="HND"):
    v = v_bits if layout == "HND" else np.ascontiguousarray(v_bits.transpose(1, 0, 2))
    desc = make_desc(w, layout)
    desc.keep_v = Tv
    dv = to_dev(v)
    packed_v = torch.empty(max(spark.packed_values_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    spark.prune_values(desc, dv, packed_v)
    mask = torch.empty((w.total, w.n_kv_heads, 4), dtype=torch.int32, device="cuda")
    vals = torch.empty((w.total, w.n_kv_heads, Tv), dtype=torch.int16, device="cuda")
    spark.unpack_values(desc, packed_v, mask, vals)
    torch.cuda.synchronize()
    return desc, packed_v, mask.cpu().numpy().view(np.uint32), vals.cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("Tv", [1, 26, 63, 64, 65, 96, 127, 128])
def test_value_selection_matches_oracle(Tv):
    w = wl.small(name=f"values{Tv}", seqlens=(130, 321), seed=200 + Tv)
    t = wl.generate(w)
    pv = oracle.prune_values(t.v, t.layout, Tv)
    print(f"{w.name}: rows={w.total * w.n_kv_heads} near-ties(<1e-6)={pv.near_ties()}")
    _, _, mask, vals = _prune_values_gpu(w, t.v, Tv)
    assert np.array_equal(mask, pv.mask)
    assert np.array_equal(vals, pv.kept)


@pytest.mark.parametrize("layout", ["HND", "NHD"])
def test_value_selection_layouts_ties_zero_rows(layout):
    w = wl.small(name=f"values_ties_{layout}", batch=2, n_q_heads=4, n_kv_heads=2, seqlens=(150, 43), seed=230)
    t = wl.generate(w)
    rng = np.random.default_rng(230)
    vq = rng.integers(-2, 3, size=t.v.shape).astype(np.float32)      # a handful of magnitudes: ties at most cuts
    vq[:, 10:20, :] = 0.0                                            # all-zero rows keep channels 0..Tv-1
    vq[:, 30:40, :] = -1.5                                           # all-equal rows
    vbits = wl.f32_to_bf16_bits(vq)
    pv = oracle.prune_values(vbits, "HND", 48)
    assert pv.near_ties() > 0.5 * pv.gap.size
    _, _, mask, vals = _prune_values_gpu(w, vbits, 48, layout)
    assert np.array_equal(mask, pv.mask)
    assert np.array_equal(vals, pv.kept)
