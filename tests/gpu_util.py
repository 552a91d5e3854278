"""Helpers shared by the GPU parity tests, the smoke check and the benchmark's checks:
upload a generated workload, run the HIP library through its C ABI, bring results back."""
from __future__ import annotations

import numpy as np
import torch

import paper_2508_15212_amd as spark


def to_dev(x: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns (or any numpy array) -> device tensor of the same bits."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda()
    return torch.from_numpy(x).cuda()


def make_desc(w, layout="HND", pack=spark.PACK_BF16, out_dtype=spark.OUT_F32, n_splits=0, total=None):
    total = w.total if total is None else total
    d = spark.SparkDesc()
    d.batch, d.n_q_heads, d.n_kv_heads, d.head_dim = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    d.keep, d.window, d.pack_dtype, d.out_dtype = w.keep, w.window, pack, out_dtype
    d.total_tokens = total
    if layout == "HND":
        d.k_token_stride = d.v_token_stride = w.head_dim
        d.k_head_stride = d.v_head_stride = total * w.head_dim
    else:
        d.k_token_stride = d.v_token_stride = w.n_kv_heads * w.head_dim
        d.k_head_stride = d.v_head_stride = w.head_dim
    d.softmax_scale = 0.0
    d.n_splits = n_splits
    return d


def run_gpu_case(w, t, layout="HND", pack=spark.PACK_BF16, n_splits=0, want_unpack=True, want_bf16=True):
    """prune -> (unpack) -> decode on the GPU.  Returns a dict of numpy arrays."""
    k, v = t.k, t.v
    if layout == "NHD":
        k = np.ascontiguousarray(k.transpose(1, 0, 2))
        v = np.ascontiguousarray(v.transpose(1, 0, 2))
    dk, dv, dqw, dq = to_dev(k), to_dev(v), to_dev(t.qwin), to_dev(t.q)
    dcu = torch.from_numpy(np.asarray(t.cu, np.int32)).cuda()
    desc = make_desc(w, layout, pack, spark.OUT_F32, n_splits)
    total, hkv, T = w.total, w.n_kv_heads, w.keep
    packed = torch.empty(max(spark.packed_bytes(desc), 256), dtype=torch.uint8, device="cuda")
    spark.prune(desc, dk, dqw, dcu, packed)
    res = {"desc": desc, "packed": packed, "dev": (dk, dv, dqw, dq, dcu)}
    if want_unpack:
        mask = torch.empty((total, hkv, 4), dtype=torch.int32, device="cuda")
        vals = torch.empty((total, hkv, T), dtype=torch.int8 if pack == spark.PACK_INT8 else torch.int16, device="cuda")
        mu = torch.empty((total, hkv), dtype=torch.float32, device="cuda")
        scale = torch.empty((total, hkv), dtype=torch.float32, device="cuda") if pack == spark.PACK_INT8 else None
        a = torch.empty((w.batch, hkv, w.head_dim), dtype=torch.float32, device="cuda")
        spark.unpack(desc, packed, mask, vals, mu, scale, a)
        res["mask"] = mask.cpu().numpy().view(np.uint32)
        res["vals"] = vals.cpu().numpy() if pack == spark.PACK_INT8 else vals.cpu().numpy().view(np.uint16)
        res["mu"] = mu.cpu().numpy()
        res["a"] = a.cpu().numpy()
        if scale is not None:
            res["scale"] = scale.cpu().numpy()
    ws = spark.new_decode_workspace(desc)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    spark.decode_attn(desc, dq, packed, dv, dcu, out, ws)
    res["out_f32"] = out.cpu().numpy()
    if want_bf16:
        desc_b = make_desc(w, layout, pack, spark.OUT_BF16, n_splits)
        outb = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device="cuda")
        spark.decode_attn(desc_b, dq, packed, dv, dcu, outb, ws)
        res["out_bf16"] = outb.float().cpu().numpy()
    torch.cuda.synchronize()
    return res
