"""The library allocates nothing, never synchronises and enqueues only kernels on the caller's stream, so a
prune + decode step can be captured into a HIP graph and replayed.  Every replay must reproduce the eager
result, with eager work and synchronisations of the program in between."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_2508_15212_amd as spark
from tests.gpu_util import make_desc, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_splits", [0, -1])
def test_prune_and_decode_replay_from_a_captured_graph(n_splits):
    """n_splits = -1: the balanced cut, whose wavefronts count in one by one (its merge takes the partials in
    slot order whatever the order of arrival, so replays are bit-identical too)."""
    w = wl.small(name="graph", batch=3, n_q_heads=8, n_kv_heads=2, keep=26, seqlens=(700, 64, 190), seed=500)
    t = wl.generate(w)
    desc = make_desc(w, n_splits=n_splits)
    dk, dv, dqw, dq = to_dev(t.k), to_dev(t.v), to_dev(t.qwin), to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    packed = torch.empty(spark.packed_bytes(desc), dtype=torch.uint8, device="cuda")
    ws = spark.new_decode_workspace(desc)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")

    def step():
        spark.prune(desc, dk, dqw, dcu, packed)
        spark.decode_attn(desc, dq, packed, dv, dcu, out, ws)

    step()
    torch.cuda.synchronize()
    eager = out.clone()
    eager_packed = packed.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for i in range(4):
        out.fill_(float("nan"))                  # eager work between replays
        packed.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(packed, eager_packed), f"replay {i}: packed cache differs"
        assert torch.equal(out, eager), f"replay {i}: decode output differs"
    # a new decode query through the same graph: inputs are read at replay time
    dq.copy_(to_dev(wl.f32_to_bf16_bits(-wl.bf16_bits_to_f32(t.q))))
    g.replay()
    torch.cuda.synchronize()
    replayed = out.clone()
    step()
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and not torch.equal(out, eager)
    assert torch.equal(out, replayed)
