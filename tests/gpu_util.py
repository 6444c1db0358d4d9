"""Helpers for the GPU parity tests: upload seeded workloads, run the HIP path through the
binding, and compare with the CPU oracle.  The oracle only ever sees the host arrays of the
workload generator and, for the integer checks, the device's own float32 logits."""
import numpy as np
import torch

import paper_2605_02960_amd as moe
import workloads
from oracle import moe_oracle as mo

DEV = "cuda:0"


def to_dev(a):
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def upload(d):
    return {k: to_dev(v) for k, v in d.items()}


def config_for(w, out_dtype=moe.DTYPE_F32, flags=0):
    xd = moe.DTYPE_F32 if w.dtype == "fp32" else moe.DTYPE_BF16
    wd = {"fp32": moe.DTYPE_F32, "bf16": moe.DTYPE_BF16, "fp8": moe.DTYPE_FP8_E4M3}[w.dtype]
    return moe.make_config(w.T, w.H, w.E, w.K, w.I, xd, wd, out_dtype, flags)


def block16_half_step(y_ref):
    """Largest error the block-scaled 16-bit storage of y may add to each element: half a code
    step of the element's 16-column block, at most amax/32768 (see MOE_FLAG_Y_F32 in the header)."""
    shp = y_ref.shape
    b = np.abs(y_ref).reshape(-1, shp[-1] // 16, 16)
    return np.repeat(b.max(axis=-1) / 32768.0, 16, axis=-1).reshape(shp)


def rms(a):
    a = np.asarray(a, dtype=np.float64)
    return float(np.sqrt(np.mean(a * a))) if a.size else 0.0


def max_err_over_rms(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref))) / max(rms(ref), 1e-300)


def run_staged(cfg, g, want_act=True):
    """The four calls in sequence; returns a dict of device tensors."""
    idx, w, logits = moe.moe_route(cfg, g["x"], g["w_router"], g["bias"])
    counts, offsets, perm, inv, _ = moe.moe_permute(cfg, idx)
    y, act, act_q, act_s = moe.moe_grouped_ffn(cfg, g["x"], perm, offsets, g["w_gate"], g["w_up"], g["w_down"],
                                               g.get("s_gate"), g.get("s_up"), g.get("s_down"), want_act=want_act)
    out = moe.moe_combine(cfg, y, inv, w)
    torch.cuda.synchronize()
    return dict(logits=logits, topk_idx=idx, topk_w=w, counts=counts, offsets=offsets, perm=perm,
                inv_perm=inv, y_perm=y, act=act, act_q=act_q, act_scale=act_s, out=out)


def check_routing_and_grouping(cfg, d, r, logit_tol=1e-4):
    """Integer outputs bit-exact against the oracle's selection on the device's own float32
    logits; logits and weights within tolerance.  Returns the oracle's routing dict."""
    l_gpu = r["logits"].cpu().numpy()
    l_ref = mo.router_logits(d["x"], d["w_router"], d["bias"])
    if l_ref.size:
        assert np.max(np.abs(l_gpu - l_ref)) <= logit_tol * rms(l_ref)
    idx_ref = mo.select_topk(l_gpu.astype(np.float64), cfg.K)
    assert np.array_equal(r["topk_idx"].cpu().numpy(), idx_ref)
    w_ref = mo.topk_weights(l_gpu.astype(np.float64), idx_ref)
    w_gpu = r["topk_w"].cpu().numpy()
    if w_ref.size:
        assert np.max(np.abs(w_gpu - w_ref)) <= 1e-6
        assert np.max(np.abs(w_gpu.astype(np.float64).sum(1) - 1.0)) <= 1e-6
    counts, offsets, perm, inv = mo.group_by_expert(idx_ref, cfg.E)
    assert np.array_equal(r["counts"].cpu().numpy(), counts)
    assert np.array_equal(r["offsets"].cpu().numpy(), offsets)
    assert np.array_equal(r["perm"].cpu().numpy(), perm)
    assert np.array_equal(r["inv_perm"].cpu().numpy(), inv)
    # share of tokens whose expert set also matches selection on the float64 logits (reported)
    idx64 = mo.select_topk(l_ref, cfg.K)
    same = float(np.mean(np.all(np.sort(idx64, 1) == np.sort(idx_ref, 1), axis=1))) if idx_ref.size else 1.0
    return dict(logits_gpu=l_gpu, same_set_as_f64=same)


def oracle_out(d, cfg, l_gpu, tokens=None, act_rounding="none", fp8=False, keep_act=False, progress=None):
    return mo.moe_layer(d["x"], d["w_router"], d["w_gate"], d["w_up"], d["w_down"], cfg.K, d["bias"],
                        act_rounding=act_rounding, fp8=fp8, tokens=tokens,
                        routing_logits=l_gpu.astype(np.float64), keep_act=keep_act, progress=progress)
