"""Per-block timeline of one decode launch on a benchmark workload (a measurement aid).

    python -m paper_2508_15212_amd.decode_timeline [--config 2] [--keep T]

Builds the packed cache of the workload, switches the library's timeline aid on (include/spark_bench.h:
thread 0 of every block files the 100 MHz wall clock at entry, at the start and the end of streaming, when its
partial state is stored and at exit, together with its tile count and hardware ids), runs a few decode
launches over rotating copies of the inputs and prints a summary of the last one as a markdown table.
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--keep", type=int, default=0)
    args = ap.parse_args()
    import paper_2508_15212_amd as spark
    import workloads as wl

    w = wl.config(args.config)
    if args.keep:
        w.keep = args.keep
    t = wl.generate(w)

    def dev(x):
        return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()

    k, qwin, q = dev(t.k), dev(t.qwin), dev(t.q)
    vs = [dev(t.v) for _ in range(2)]
    cu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    d = spark.SparkDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    d.keep, d.window, d.pack_dtype, d.out_dtype = w.keep, w.window, spark.PACK_BF16, spark.OUT_BF16
    d.total_tokens = w.total
    d.k_token_stride = d.v_token_stride = w.head_dim
    d.k_head_stride = d.v_head_stride = w.total * w.head_dim
    packs = [torch.empty(spark.packed_bytes(d), dtype=torch.uint8, device="cuda") for _ in range(2)]
    for p in packs:
        spark.prune(d, k, qwin, cu, p)
    ws = spark.new_decode_workspace(d)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device="cuda")
    max_blocks = 1 << 16
    buf = torch.zeros(max_blocks * 8, dtype=torch.int64, device="cuda")
    spark.decode_timeline(buf)
    try:
        for i in range(7):                       # the last launch is the one that is read
            buf.zero_()
            spark.decode_attn(d, q, packs[i % 2], vs[i % 2], cu, out, ws)
        torch.cuda.synchronize()
    finally:
        spark.decode_timeline(None)
    tr = buf.cpu().numpy().reshape(-1, 8)
    launched = int((tr[:, 0] != 0).sum())
    tr = tr[(tr[:, 0] != 0) & (tr[:, 4] != 0)]    # (blocks past the last chunk of a ragged batch leave at once)
    us = lambda ticks: np.asarray(ticks, np.float64) / 100.0
    t00 = tr[:, 0].min()
    balanced = bool((tr[:, 5] >> 32).any())       # (the balanced cut: words are wavefront 0's, tiles its own)
    nts = tr[:, 5] & 0xFFFFFFFF
    tr = tr[nts > 0] if balanced else tr           # (wavefronts without a tile only look after empty sequences)
    nts = tr[:, 5] & 0xFFFFFFFF
    rounds = np.maximum(1, nts if balanced else (nts + 3) // 4)
    per_round = us(tr[:, 2] - tr[:, 1]) / rounds
    pct = lambda x, ps: "  /  ".join("%.1f" % v for v in np.percentile(x, ps))
    xcc = (tr[:, 6] >> 32) & 0xF
    merged = tr[:, 7] == 1
    print(f"## {w.name}, T = {w.keep}: {len(tr)} working blocks of {launched} launched, " +
          ("balanced cut (figures are those of each block's first wavefront)\n" if balanced else
           f"{spark.decode_splits(d)} chunk(s) per average sequence\n"))
    print("| quantity | value |\n|---|---|")
    print(f"| kernel span (first entry to last exit) | {us(tr[:, 4].max() - t00):.1f} us |")
    print(f"| tiles per {'wavefront' if balanced else 'block'}, min / mean / max | {nts.min()} / {nts.mean():.1f} / {nts.max()} |")
    print(f"| entry -> start of streaming, p10 / p50 / p90 (us) | {pct(us(tr[:, 1] - tr[:, 0]), [10, 50, 90])} |")
    print(f"| one round of tiles per wavefront, p10 / p50 / p90 (us) | {pct(per_round, [10, 50, 90])} |")
    print(f"| end of streaming after the first entry, p10 / p50 / p90 / max (us) | {pct(us(tr[:, 2] - t00), [10, 50, 90, 100])} |")
    if balanced:
        print(f"| end of streaming -> exit, wavefronts that merged no pair / merged one, mean (us) | "
              f"{us(tr[:, 4] - tr[:, 2])[~merged].mean():.1f} / {us(tr[:, 4] - tr[:, 2])[merged].mean() if merged.any() else 0.0:.1f} |")
    else:
        print(f"| end of streaming -> partial stored (wait for the block's slowest wavefront, reduce), p50 / p90 (us) | {pct(us(tr[:, 3] - tr[:, 2]), [50, 90])} |")
        if merged.any():
            print(f"| partial stored -> merged output written, blocks that merged ({int(merged.sum())}), mean (us) | {us(tr[:, 4] - tr[:, 3])[merged].mean():.1f} |")
    print("| round time by XCC id, mean (us) | " + ", ".join(f"{x}: {per_round[xcc == x].mean():.2f}" for x in sorted(set(xcc.tolist()))) + " |")
    groups = [(0, 4), (4, 5), (5, 6), (6, 8)] if balanced else [(0, 8), (8, 16), (16, 24), (24, 40), (40, 1 << 30)]
    for lo, hi in groups:
        m = (nts > lo) & (nts <= hi)
        if m.any() and not m.all():
            print(f"| blocks with {lo + 1}..{min(hi, int(nts.max()))} tiles: count, mean / max exit time (us) | {int(m.sum())}, "
                  f"{us(tr[:, 4] - t00)[m].mean():.1f} / {us(tr[:, 4] - t00)[m].max():.1f} |")
    print()
    return 0


if __name__ == "__main__":
    sys.exit(main())
