"""GPU test of the one-GPU weight-streaming call: layers whose expert weights are streamed from
pinned host memory through a ring of device slots must give bit-identical outputs to the same
layers run with resident weights (whose parity against the oracle test_gpu_parity.py covers)."""
import numpy as np
import pytest
import torch

import paper_2605_02960_amd as moe
import workloads
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _align(n, a=256):
    return (n + a - 1) // a * a


def _pinned(t):
    h = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
    h.copy_(t)
    return h


@pytest.mark.parametrize("dtype,n_slots,n_resident", [("bf16", 2, 0), ("bf16", 2, 1), ("bf16", 3, 2), ("bf16", 1, 0),
                                                      ("fp8", 2, 1)])
def test_streamed_layers_equal_resident_layers(dtype, n_slots, n_resident):
    base = workloads.QWEN3_8K if dtype == "bf16" else workloads.QWEN3_32K_FP8
    w = workloads.scaled(base, name=f"stream_{dtype}", T=300, H=256, E=8, K=2, I=256)
    L = 5
    cfg = gu.config_for(w)
    print(f"case stream {dtype} slots={n_slots} resident={n_resident}", flush=True)
    x = None
    layers, direct = [], []
    for i in range(L):
        g = gu.upload(workloads.generate(w, seed=i))
        if x is None:
            x = g["x"]
        if dtype == "fp8":
            for name, rows, cols in (("w_gate", w.E * w.I, w.H), ("w_up", w.E * w.I, w.H), ("w_down", w.E * w.H, w.I)):
                q, s = moe.moe_quantize_rows_e4m3(g[name].reshape(rows, cols))
                g[name], g["s_" + name[2:]] = q, s
        torch.cuda.synchronize()
        direct.append(moe.moe_prefill_layer(cfg, x, g["w_router"], None, g["w_gate"], g["w_up"], g["w_down"],
                                            g.get("s_gate"), g.get("s_up"), g.get("s_down")))
        lay = dict(w_router=g["w_router"], bias=None, out=torch.full((w.T, w.H), float("nan"), device=gu.DEV))
        for name in ("w_gate", "w_up", "w_down", "s_gate", "s_up", "s_down"):
            if name in g:
                lay[name] = _pinned(g[name].cpu())
        lay["_dev"] = g
        layers.append(lay)
    torch.cuda.synchronize()
    nbytes = moe.moe_layer_weight_bytes(cfg)
    parts = ["w_gate", "w_up", "w_down"] + (["s_gate", "s_up", "s_down"] if dtype == "fp8" else [])
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
