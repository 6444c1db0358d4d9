"""GPU tests of the one-GPU weight-streaming call (App. B.1 of the paper; the offloading pipeline
of Sec. 6.3): the expert weights of every layer are streamed from pinned host memory through a
ring of device slots.  Every streamed layer's output is compared with the CPU oracle evaluated on
that layer's own weights (routing taken on the device's float32 logits, as in the block tests),
and, as a second check, must equal bit for bit the same layer run with resident weights."""
import numpy as np
import pytest
import torch

import paper_2605_02960_amd as moe
import workloads
from oracle import moe_oracle as mo
import gpu_util as gu

pytestmark = pytest.mark.gpu

TOL_BF16_PURE = 2e-2     # float32 result against the oracle without intermediate rounding
TOL_BF16_RP = 5e-3       # against the oracle that rounds the activation to bf16
TOL_FP8 = 6e-2           # against the quantising oracle


def _align(n, a=256):
    return (n + a - 1) // a * a


def _pinned(t):
    h = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    h.copy_(t)
    return h


@pytest.mark.parametrize("dtype,n_slots,n_resident", [("bf16", 2, 0), ("bf16", 2, 1), ("bf16", 3, 2), ("bf16", 1, 0),
                                                      ("fp8", 2, 1)])
def test_streamed_layers_against_the_oracle(dtype, n_slots, n_resident):
    fp8 = dtype == "fp8"
    base = workloads.QWEN3_32K_FP8 if fp8 else workloads.QWEN3_8K
    # fp8: contractions long enough (1024 and 2048 terms) for the end-to-end bound to be meaningful
    shape = dict(T=128, H=1024, E=4, K=2, I=2048) if fp8 else dict(T=300, H=256, E=8, K=2, I=256)
    w = workloads.scaled(base, name=f"stream_{dtype}", **shape)
    L = 5
    cfg = gu.config_for(w)
    print(f"case stream {dtype} slots={n_slots} resident={n_resident}", flush=True)
    x = None
    host, layers, direct, logits = [], [], [], []
    for i in range(L):
        d = workloads.generate(w, seed=i)
        g = gu.upload(d)
        if x is None:
            x, x_host = g["x"], d["x"]
        if fp8:
            for name, rows, cols in (("w_gate", w.E * w.I, w.H), ("w_up", w.E * w.I, w.H), ("w_down", w.E * w.H, w.I)):
                q, s = moe.moe_quantize_rows_e4m3(g[name].reshape(rows, cols))
                g[name], g["s_" + name[2:]] = q, s
        torch.cuda.synchronize()
        direct.append(moe.moe_prefill_layer(cfg, x, g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"],
                                            g.get("s_gate"), g.get("s_up"), g.get("s_down")))
        logits.append(moe.moe_route(cfg, x, g["w_router"], None)[2].cpu().numpy())
        lay = dict(w_router=g["w_router"], bias=None, out=torch.full((w.T, w.H), float("nan"), device=gu.DEV))
        for name in ("w_gate", "w_up", "w_down", "s_gate", "s_up", "s_down"):
            if name in g:
                lay[name] = _pinned(g[name].cpu())
        lay["_dev"] = g
        layers.append(lay)
        host.append(d)
    torch.cuda.synchronize()
    nbytes = moe.moe_layer_weight_bytes(cfg)
    parts = ["w_gate", "w_up", "w_down"] + (["s_gate", "s_up", "s_down"] if fp8 else [])
    sizes = [layers[0][p].numel() * layers[0][p].element_size() for p in parts]
    assert nbytes == sum(_align(s) for s in sizes)
    slots = [torch.zeros(nbytes, dtype=torch.uint8, device=gu.DEV) for _ in range(n_slots)]
    for j in range(n_resident):          # resident layers: laid out as the call lays them out
        off = 0
        for p, s in zip(parts, sizes):
            slots[j][off:off + s] = layers[j]["_dev"][p].reshape(-1).view(torch.uint8)
            off += _align(s)
    torch.cuda.synchronize()
    pairs = moe.moe_prefill_layers_streamed(cfg, layers, x, slots, n_resident=n_resident, time_layers=True)
    torch.cuda.synchronize()
    ev = moe.HipEvents()
    for i in range(L):
        d = host[i]
        out = layers[i]["out"].cpu().numpy()
        # the oracle on layer i's own weights (the layers share x), routed on the device's logits
        kw = dict(routing_logits=logits[i].astype(np.float64))
        if fp8:
            ref = mo.moe_layer(x_host, d["w_router"], d["w_gate"], d["w_up"], d["w_down"], w.K, None, fp8=True, **kw)
            e = gu.max_err_over_rms(out, ref["out"])
            print(f"  layer {i}: max|err|/rms vs quantising oracle {e:.3e}", flush=True)
            assert e <= TOL_FP8, f"layer {i}"
        else:
            pure = mo.moe_layer(x_host, d["w_router"], d["w_gate"], d["w_up"], d["w_down"], w.K, None, **kw)
            rp = mo.moe_layer(x_host, d["w_router"], d["w_gate"], d["w_up"], d["w_down"], w.K, None,
                              act_rounding="bf16", **kw)
            e_pure, e_rp = gu.max_err_over_rms(out, pure["out"]), gu.max_err_over_rms(out, rp["out"])
            print(f"  layer {i}: max|err|/rms vs unrounded oracle {e_pure:.3e}, vs bf16-activation oracle {e_rp:.3e}",
                  flush=True)
            assert e_pure <= TOL_BF16_PURE and e_rp <= TOL_BF16_RP, f"layer {i}"
        # a layer's weights must not leak into its neighbour's slot: the wrong layer's oracle is far away
        if i > 0:
            other = mo.moe_layer(x_host, host[i - 1]["w_router"], host[i - 1]["w_gate"], host[i - 1]["w_up"],
                                 host[i - 1]["w_down"], w.K, None, fp8=fp8)
            assert gu.max_err_over_rms(out, other["out"]) > 0.5
        # second check: streamed == resident, bit for bit
        assert torch.equal(layers[i]["out"], direct[i]), f"layer {i}"
        assert ev.elapsed_ms(*pairs[i]) > 0


def test_streamed_argument_errors():
    w = workloads.scaled(workloads.QWEN3_8K, T=64, H=256, E=8, K=2, I=256)
    cfg = gu.config_for(w)
    g = gu.upload(workloads.generate(w))
    lay = dict(w_router=g["w_router"], bias=None, out=torch.empty((w.T, w.H), device=gu.DEV),
               w_gate=_pinned(g["w_gate"].cpu()), w_up=_pinned(g["w_up"].cpu()), w_down=_pinned(g["w_down"].cpu()))
    slots = [torch.zeros(moe.moe_layer_weight_bytes(cfg), dtype=torch.uint8, device=gu.DEV)]
    s = torch.cuda.current_stream()
    with pytest.raises(moe.MoEError) as e:
        moe.moe_prefill_layers_streamed(cfg, [lay], g["x"], slots, compute_stream=s, copy_stream=s)
    assert e.value.status == -6          # the two streams must differ
    with pytest.raises(moe.MoEError) as e:
        moe.moe_prefill_layers_streamed(cfg, [lay], g["x"], slots, n_resident=2)
    assert e.value.status == -2
    with pytest.raises(moe.MoEError) as e:
        moe.moe_prefill_layers_streamed(cfg, [dict(lay, w_up=None)], g["x"], slots)
    assert e.value.status == -1
