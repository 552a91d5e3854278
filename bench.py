#!/usr/bin/env python3
"""Benchmark of the SparK hot path on one MI355X.

A step is one pass of the whole path over one batch of seeded synthetic input that is
already resident in HBM: spark_prune (window statistic, saliency, per-token top-T, pack)
followed by spark_decode_attn (query prep, recovered scores, online softmax, P V, combine).
The headline value is the decode-attention time per step on the Llama-3.1-8B-shaped
configuration (batch 8, 32 q / 8 kv heads, head_dim 128, 32K context, 26 of 128 channels
kept), with the achieved fraction of the HBM roofline beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-cpu]

Prints ONE JSON line.  `value` is the decode time inside the prune + decode step (an event
between the two phases); `roofline` prices the decode kernel's algorithmic bytes against 8 TB/s
using the kernel's average duration over the same number of back-to-back launches, also by HIP
events inside this run, and carries the HBM traffic that the byte counters of a profiler run
measured for the workload (read from the profile summary that `traffic_source` names);
`cpu_baseline` is the CPU oracle timed on this host (context only, and the one place this file
touches `oracle/`).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM bytes per decode launch measured with rocprofv3 --pmc (FETCH_SIZE x its calibration factor + WRITE_SIZE), per
# (workload, pack).  Each entry names the profile summary that holds the counter readings and the line
# "traffic_bytes[workload,pack] = N" this file reads; a workload with no entry (or a variant the counters were
# not taken for) reports null.  These are stored measurements: they move when the profile is taken again, not
# when the kernel changes.
TRAFFIC_PROFILES = {
    ("cfg2_llama8b_b8_32k_keep26", "bf16"): "profiles/decode_prune_cfg2_hbm_traffic.md",
    ("cfg2_llama8b_b8_32k_keep26", "int8"): "profiles/decode_prune_cfg2_hbm_traffic.md",
    ("cfg3_prune_131k", "bf16"): "profiles/decode_prune_cfg3_hbm_traffic.md",
    ("cfg4_ragged_b64_keep64", "bf16"): "profiles/decode_prune_cfg4_hbm_traffic.md",
    ("cfg5_qwen32b_b4_131k_keep26", "bf16"): "profiles/decode_prune_cfg5_hbm_traffic.md",
}


def measured_traffic(workload: str, pack: str):
    """(bytes, profile file) of the stored HBM-counter measurement for this workload, or (None, None)."""
    rel = TRAFFIC_PROFILES.get((workload, pack))
    if rel is None:
        return None, None
    key = "traffic_bytes[%s,%s] = " % (workload, pack)
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                if line.strip().startswith(key):
                    return int(line.strip()[len(key):]), rel
    except OSError:
        pass
    return None, None


def device_state(torch) -> dict:
    """Name, size and clocks of the GPU the run used (the clocks as rocm-smi reports them after the run, if it can
    be asked; a reading that fails is left out rather than guessed)."""
    import subprocess
    p = torch.cuda.get_device_properties(0)
    dev = {"name": p.name, "compute_units": p.multi_processor_count, "memory_GiB": round(p.total_memory / 2 ** 30, 1),
           "max_engine_clock_MHz": round(getattr(p, "clock_rate", 0) / 1e3) or None,
           "max_memory_clock_MHz": round(getattr(p, "memory_clock_rate", 0) / 1e3) or None, "rocm_smi": None}
    try:
        out = subprocess.run(["rocm-smi", "-d", "0", "--showclocks", "--showperflevel", "--showpower", "--json"],
                             capture_output=True, text=True, timeout=15)
        if out.returncode == 0 and out.stdout.strip().startswith("{"):
            card = next(iter(json.loads(out.stdout).values()))
            dev["rocm_smi"] = {k: v for k, v in card.items()
                               if any(t in k.lower() for t in ("sclk", "mclk", "fclk", "performance level", "power"))}
    except Exception:
        pass
    return {k: v for k, v in dev.items() if v is not None}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="workload 1..5 (2 = the headline metric)")
    ap.add_argument("--keep", type=int, default=0, help="override T")
    ap.add_argument("--int8", action="store_true", help="int8 storage of the kept entries")
    ap.add_argument("--keep-v", type=int, default=0,
                    help="also prune the value cache to this many channels per row (0 = values stay dense)")
    ap.add_argument("--recovery", choices=["degenerate", "gaussian", "exponential"], default="degenerate",
                    help="recovery function at decode (the sampled ones store two more statistics per row)")
    ap.add_argument("--top-p", type=int, default=0,
                    help="the top-p variant: keep per row the fewest channels holding this many basis points of the "
                         "row's saliency (9900 = 99 %%); prune through spark_prune_topp, decode through spark_decode_attn_topp")
    ap.add_argument("--tail", type=int, default=0,
                    help="appended never-pruned rows per sequence (decode through spark_decode_attn_tail)")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--copies", type=int, default=4, help="input copies rotated to defeat the 256 MB cache")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--decode-only", action="store_true", help="time decode alone (profiling aid)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is a one-GPU hot path; it has no multi-GPU mode (run with --gpus 1)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2508_15212_amd as spark
    import workloads as wl

    spark.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    w = wl.config(args.config)
    if args.keep:
        w.keep = args.keep
    if args.top_p:
        # keys whose magnitude sits in a minority of channels, as in real key caches: with these two figures a
        # 99 % threshold drops 58 % of the channels on average, the overall ratio the paper reports for the variant
        w.quiet_fraction, w.quiet_scale = 0.6, 0.008
        w.name += "_quiet60"
    pack = spark.PACK_INT8 if args.int8 else spark.PACK_BF16
    t0 = time.time()
    t = wl.generate(w)
    gen_s = time.time() - t0

    def dev(x):
        return torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()

    total, hkv, hq, D, T = w.total, w.n_kv_heads, w.n_q_heads, w.head_dim, w.keep
    desc = spark.SparkDesc()
    desc.batch, desc.n_q_heads, desc.n_kv_heads, desc.head_dim = w.batch, hq, hkv, D
    desc.keep, desc.window, desc.pack_dtype, desc.out_dtype = T, w.window, pack, spark.OUT_BF16
    desc.total_tokens = total
    desc.k_token_stride = desc.v_token_stride = D
    desc.k_head_stride = desc.v_head_stride = total * D
    desc.n_splits = args.splits
    desc.max_seqlen = int(np.max(np.diff(np.asarray(t.cu, np.int64))))     # (a serving engine knows its batch)
    desc.keep_v = args.keep_v
    Tv = args.keep_v
    ntail = args.tail
    desc.tail_capacity = ntail
    rec = {"degenerate": 0, "gaussian": spark.RECOVER_GAUSSIAN, "exponential": spark.RECOVER_EXPONENTIAL}[args.recovery]
    desc.stats = 1 if rec else 0
    rec_seed = 0x5EED0000 + w.seed
    if rec and (Tv or ntail or args.int8):
        print("bench.py: --recovery gaussian/exponential is timed on its own (no --keep-v / --tail / --int8)",
              file=sys.stderr)
        return 2
    if ntail and Tv:
        print("bench.py: --tail and --keep-v are separate entry points; pick one", file=sys.stderr)
        return 2
    topp = args.top_p
    if topp and (Tv or ntail or rec or args.int8 or args.keep):
        print("bench.py: --top-p is timed on its own (no --keep / --keep-v / --tail / --recovery / --int8)", file=sys.stderr)
        return 2

    ncopy = max(1, args.copies)
    k0, v0 = dev(t.k), dev(t.v)
    ks = [k0] + [k0.clone() for _ in range(ncopy - 1)]
    vs = [v0] + [v0.clone() for _ in range(ncopy - 1)]
    qwin, q = dev(t.qwin), dev(t.q)
    cu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    pbytes = spark.packed_topp_bytes(desc) if topp else spark.packed_bytes(desc)
    packs = [torch.empty(pbytes, dtype=torch.uint8, device="cuda") for _ in range(ncopy)]
    packvs = ([torch.empty(spark.packed_values_bytes(desc), dtype=torch.uint8, device="cuda") for _ in range(ncopy)]
              if Tv else None)
    ws = spark.new_decode_workspace(desc)
    out = torch.empty((w.batch, hq, D), dtype=torch.bfloat16, device="cuda")

    def prune_all(c):
        if topp:
            spark.prune_topp(desc, ks[c], qwin, cu, topp, packs[c])
            return
        spark.prune(desc, ks[c], qwin, cu, packs[c])
        if Tv:
            spark.prune_values(desc, vs[c], packvs[c])

    if ntail:
        rng = np.random.default_rng(w.seed + 7)
        tshape = (w.batch, ntail, hkv, D)
        tail_k_np = wl.f32_to_bf16_bits(rng.standard_normal(tshape).astype(np.float32))
        tail_v_np = wl.f32_to_bf16_bits(rng.standard_normal(tshape).astype(np.float32))
        tail_len_np = np.full(w.batch, ntail, np.int32)
        tail_k, tail_v = dev(tail_k_np), dev(tail_v_np)
        tail_len = torch.from_numpy(tail_len_np).cuda()

    def decode(c, d=desc, o=out):
        if topp:
            spark.decode_attn_topp(d, q, packs[c], vs[c], cu, o, ws)
        elif rec:
            spark.decode_attn_sampled(d, q, packs[c], vs[c], cu, o, ws, rec, rec_seed)
        elif ntail:
            spark.decode_attn_tail(d, q, packs[c], vs[c], cu, tail_k, tail_v, tail_len, o, ws)
        elif Tv:
            spark.decode_attn_values(d, q, packs[c], packvs[c], cu, o, ws)
        else:
            spark.decode_attn(d, q, packs[c], vs[c], cu, o, ws)

    for c in range(ncopy):
        prune_all(c)
    torch.cuda.synchronize()

    def step(i, ev=None):
        c = i % ncopy
        if ev is not None:
            ev[0].record()
        if not args.decode_only:
            prune_all(c)
        if ev is not None:
            ev[1].record()
        decode(c)
        if ev is not None:
            ev[2].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prune_ms = np.array([e[0].elapsed_time(e[1]) for e in evs])
    dec_ms = np.array([e[1].elapsed_time(e[2]) for e in evs])

    # The decode kernel's own average duration: the same launches back to back between one pair of events
    # (the per-step figure above also contains the gap that the event between prune and decode opens).
    ka, kb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(min(args.warmup, 3)):
        decode(i % ncopy)
    ka.record()
    for i in range(args.steps):
        decode(i % ncopy)
    kb.record()
    torch.cuda.synchronize()
    kern_us = float(ka.elapsed_time(kb) * 1e3 / max(1, args.steps))

    # Streaming-read yardstick on this machine: the library's plain read kernel over one V copy
    # (also the kernel of known size that scales the HBM byte counters of a profiler run).
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    probe_blocks = 512      # two blocks per compute unit: the fastest plain read on this part (more are slower)
    for c in range(ncopy):
        spark.probe_read(vs[c], sink, probe_blocks)
    torch.cuda.synchronize()
    pev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(9)]
    for i, (a, b) in enumerate(pev):
        a.record()
        spark.probe_read(vs[i % ncopy], sink, probe_blocks)
        b.record()
    torch.cuda.synchronize()
    probe_us = float(np.median([a.elapsed_time(b) for a, b in pev]) * 1e3)
    probe_bytes = vs[0].numel() * vs[0].element_size()
    probe_gbs = probe_bytes / (probe_us * 1e-6) / 1e9

    rows = total * hkv
    row_bytes = (pbytes - 256 - 2 * ((w.batch * hkv * D * 4 + 255) // 256 * 256)) / (
        hkv * ((total + 63) // 64) * 64)
    k_row = (T + 16 + 4 + 4) if args.int8 else (2 * T + 16 + 4)      # kept entries + mask + mu (+ scale)
    mean_kept = None
    if topp:
        # rows of 24 bytes (mask, mu, count) plus the kept entries, every row rounded up to a whole 4-byte word
        cnt = torch.empty((total, hkv), dtype=torch.int32, device="cuda")
        spark.unpack_topp(desc, packs[0], None, cnt, None, None, None)
        mean_kept = float(cnt.float().mean().item())
        k_row = 24 + 4.0 * float(((cnt + 1) // 2).float().mean().item())
        row_bytes = k_row
    if rec:
        k_row += 8                                                    # all-channel mean and standard deviation
    v_row = (2 * Tv + 16) if Tv else 2 * D                            # kept entries + mask, or the dense row
    dec_alg_bytes = rows * (k_row + v_row)                            # packed K row + V row
    dec_alg_bytes += w.batch * ntail * hkv * 4 * D                    # appended rows: dense K and V
    prune_alg_bytes = rows * (2 * D + k_row) + w.batch * hq * w.window * D * 2
    if Tv:
        prune_alg_bytes += rows * (2 * D + v_row)
    dec_us = float(dec_ms.mean() * 1e3)
    prune_us = float(prune_ms.mean() * 1e3)
    dec_gbs = dec_alg_bytes / (dec_us * 1e-6) / 1e9
    kern_gbs = dec_alg_bytes / (kern_us * 1e-6) / 1e9
    prune_gbs = prune_alg_bytes / (prune_us * 1e-6) / 1e9 if prune_us > 0 else 0.0

    traffic_bytes, traffic_file = (None, None)
    if not (args.keep or Tv or ntail or rec or topp):
        traffic_bytes, traffic_file = measured_traffic(w.name, "int8" if args.int8 else "bf16")

    result = {
        "metric": "decode-attn \u00b5s/step + achieved HBM GB/s (% peak) at 32K ctx, 80% prune",
        "value": round(dec_us, 2),
        "unit": "\u00b5s/step (decode attention)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": w.name, "batch": w.batch, "n_q_heads": hq, "n_kv_heads": hkv, "head_dim": D,
            "context": int(w.seqlens.max()), "total_tokens": total, "keep": T, "window": w.window,
            "pack": "int8" if args.int8 else "bf16", "keep_v": Tv if Tv else None, "tail_rows_per_sequence": ntail if ntail else None,
            "recovery": args.recovery, "top_p_basis_points": topp if topp else None,
            "mean_kept_per_row": mean_kept,
            "splits": spark.decode_splits(desc),       # (0: the balanced cut, tiles dealt out to wavefronts)
            "input_copies_rotated": ncopy, "seed": w.seed, "step": ("spark_prune + spark_prune_values + spark_decode_attn_values" if Tv
                                                              else "spark_prune_topp + spark_decode_attn_topp" if topp
                                                              else "spark_prune + spark_decode_attn_tail" if ntail
                                                              else "spark_prune + spark_decode_attn"),
        },
        # two decode figures: "decode" = HIP events around spark_decode_attn inside the prune + decode step (what
        # `value` reports; includes the launch gap after the prune kernel); "roofline" = the decode kernel alone,
        # launched back to back (what `roofline.frac` prices)
        "decode": {"timed": "inside the prune + decode step", "us_mean": round(dec_us, 2), "us_min": round(float(dec_ms.min() * 1e3), 2),
                   "us_median": round(float(np.median(dec_ms) * 1e3), 2),
                   "algorithmic_MB": round(dec_alg_bytes / 1e6, 1), "GBps": round(dec_gbs, 1),
                   "in_step_pct_of_8TBps": round(100 * dec_gbs / HBM_PEAK_GBS, 1)},
        "prune": {"us_mean": round(prune_us, 2), "us_min": round(float(prune_ms.min() * 1e3), 2),
                  "algorithmic_MB": round(prune_alg_bytes / 1e6, 1), "GBps": round(prune_gbs, 1),
                  "pct_of_8TBps": round(100 * prune_gbs / HBM_PEAK_GBS, 1),
                  "Mtokens_per_s": round(total / prune_us, 2) if prune_us > 0 else None},
        "roofline": {"bound": "hbm", "achieved": round(kern_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(kern_gbs / HBM_PEAK_GBS, 4),
                     "kernel_us": round(kern_us, 2),
                     "traffic": traffic_bytes, "traffic_source": traffic_file,
                     "algorithmic_bytes": dec_alg_bytes,
                     "kernel": "spark_decode_kernel, HIP events around %d back-to-back launches" % args.steps},
        "stream_read_ceiling": {"GBps": round(probe_gbs, 1), "us": round(probe_us, 2),
                                "MB": round(probe_bytes / 1e6, 1),
                                "decode_pct_of_ceiling": round(100 * kern_gbs / probe_gbs, 1),
                                "kernel": "spark_probe_read_kernel, %d blocks" % probe_blocks},
        "packed_row_bytes": row_bytes,
        "input_generation_s": round(gen_s, 1),
    }

    if not args.no_cpu:
        # CPU baseline: the oracle as it stands, on this host's cores, one pass over the same workload.
        import oracle
        threads = oracle.max_threads()
        t0 = time.perf_counter()
        _, _, a32 = oracle.window_stat(t.qwin, hkv)
        pr = oracle.prune_topp(t.k, t.layout, a32, t.cu, topp) if topp else oracle.prune(t.k, t.layout, a32, t.cu, T)
        if args.int8:
            pr = oracle.quant_int8(pr)
        t1 = time.perf_counter()
        if Tv:
            pv = oracle.prune_values(t.v, t.layout, Tv)
            t1 = time.perf_counter()
            ref = oracle.decode_literal(t.q, pr, oracle.expand_values(pv), "NHD", t.cu)
        elif rec:
            mu_all, sigma_all = oracle.row_stats(t.k, t.layout, a32, t.cu)
            t1 = time.perf_counter()
            ref = oracle.decode_sampled(rec, rec_seed, t.q, pr, mu_all, sigma_all, t.v, t.layout, t.cu)
        elif ntail:
            ref = oracle.decode_literal_tail(t.q, pr, t.v, t.layout, t.cu, tail_k_np, tail_v_np, tail_len_np)
        else:
            ref = oracle.decode_literal(t.q, pr, t.v, t.layout, t.cu)
        t2 = time.perf_counter()
        result["cpu_baseline"] = {
            "value": round((t2 - t1) * 1e6, 0), "unit": "us/step (decode attention)", "cores": threads,
            "kind": "oracle", "sample": "the full workload, one pass (prune %.2f s, decode %.2f s)" % (t1 - t0, t2 - t1),
            "prune_us": round((t1 - t0) * 1e6, 0),
        }
        # the oracle's result is at hand: compare the last GPU step against it
        c = (args.steps - 1) % ncopy if args.steps > 0 else 0
        mask = torch.empty((total, hkv, 4), dtype=torch.int32, device="cuda")
        if topp:
            spark.unpack_topp(desc, packs[c], mask, None, None, None, None)
        else:
            spark.unpack(desc, packs[c], mask, None, None, None, None)
        desc32 = spark.SparkDesc.from_buffer_copy(desc)
        desc32.out_dtype = spark.OUT_F32
        out32 = torch.empty((w.batch, hq, D), dtype=torch.float32, device="cuda")
        decode(c, desc32, out32)
        torch.cuda.synchronize()
        err = np.abs(out32.cpu().numpy().astype(np.float64) - ref)
        if Tv:
            mask_v = torch.empty((total, hkv, 4), dtype=torch.int32, device="cuda")
            spark.unpack_values(desc, packvs[c], mask_v, None)
            result["value_masks_bit_exact"] = bool(np.array_equal(mask_v.cpu().numpy().view(np.uint32), pv.mask))
        result["parity"] = {"masks_bit_exact": bool(np.array_equal(mask.cpu().numpy().view(np.uint32), pr.mask)),
                            "near_tie_rows_gap_lt_1e-6": pr.near_ties(), "rows": int(rows),
                            "decode_max_abs_err": float(err.max()), "decode_mean_abs_err": float(err.mean())}

    result["device"] = device_state(torch)
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
