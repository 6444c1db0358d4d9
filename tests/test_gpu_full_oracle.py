"""Full-size parity, every token: the fused call at the three large configurations (235B-A22B
layer shape: T = 8192 bf16, T = 65536 bf16 with Zipf-like routing, T = 32768 fp8) against the CPU
oracle evaluated for ALL tokens, not a sample.  The two bf16 configurations take about a minute
together on 16 host cores and always run; the fp8 one (the oracle quantises all 384 expert
matrices: two minutes, silent under a quiet test runner) runs when MOE_FULL_ORACLE=1 is set, and
the default suite checks it on sampled tokens.  Measured values are recorded in the design notes."""
import os
import time

import numpy as np
import pytest
import torch

import paper_2605_02960_amd as moe
import workloads
from oracle import moe_oracle as mo
import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("w", [workloads.QWEN3_8K, workloads.QWEN3_64K_ZIPF, workloads.QWEN3_32K_FP8], ids=lambda w: w.name)
def test_every_token_against_the_oracle(w):
    fp8 = w.dtype == "fp8"
    if fp8 and os.environ.get("MOE_FULL_ORACLE") != "1":
        pytest.skip("set MOE_FULL_ORACLE=1 (two minutes of host time without output)")
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    scales = {}
    if fp8:
        for name, rows, cols in (("w_gate", w.E * w.I, w.H), ("w_up", w.E * w.I, w.H), ("w_down", w.E * w.H, w.I)):
            g[name], scales["s_" + name[2:]] = moe.moe_quantize_rows_e4m3(g[name].reshape(rows, cols))
    taps = dict(logits=torch.empty((w.T, w.E), dtype=torch.float32, device=gu.DEV),
                topk_idx=torch.empty((w.T, w.K), dtype=torch.int32, device=gu.DEV),
                topk_w=torch.empty((w.T, w.K), dtype=torch.float32, device=gu.DEV),
                counts=torch.empty((w.E,), dtype=torch.int32, device=gu.DEV),
                offsets=torch.empty((w.E + 1,), dtype=torch.int32, device=gu.DEV),
                perm=torch.empty((w.rows,), dtype=torch.int32, device=gu.DEV),
                inv_perm=torch.empty((w.rows,), dtype=torch.int32, device=gu.DEV))
    out = moe.moe_prefill_layer(cfg, g["x"], g["w_router"], g["bias"], g["w_gate"], g["w_up"], g["w_down"],
                                scales.get("s_gate"), scales.get("s_up"), scales.get("s_down"), taps=taps)
    torch.cuda.synchronize()
    r = dict(taps, out=out)
    info = gu.check_routing_and_grouping(cfg, d, r)          # integer outputs in full, as in the default suite
    out_h = out.cpu().numpy()
    del g, taps, r
    torch.cuda.empty_cache()
    print(f"case {w.name}: oracle over all {w.T} tokens", flush=True)
    for flavour in (("fp8",) if fp8 else ("pure", "bf16_act")):
        t0 = time.time()
        def progress(e, t0=t0):
            if e % 8 == 7:
                print(f"    oracle [{flavour}]: expert {e + 1} of {w.E} done, {time.time() - t0:.0f} s", flush=True)

        ref = gu.oracle_out(d, cfg, info["logits_gpu"], tokens=None, fp8=fp8,
                            act_rounding="bf16" if flavour == "bf16_act" else "none", progress=progress)["out"]
        err = np.abs(out_h - ref)
        rms = gu.rms(ref)
        e = float(err.max()) / rms
        # Against the oracle that rounds the activation to bf16 the distance is set by single
        # activations that land on the other side of a bf16 rounding boundary (one ulp); over all
        # 2.7e8 outputs of the 64K-token batch the largest such case is a token whose first expert
        # carries a combine weight of 0.87 (measured 1.0e-2 * rms), so the sampled-token bound of
        # the default suite (5e-3) does not apply here: both bf16 flavours are held to 2e-2.
        bound = {"fp8": 6e-2, "pure": 2e-2, "bf16_act": 2e-2}[flavour]
        e_rms = float(np.sqrt(np.mean(err * err))) / rms
        per_token = err.max(axis=1) / rms
        over = np.flatnonzero(per_token > bound)
        print(f"  {w.name} [{flavour}]: max|err|/rms over all tokens = {e:.3e} (bound {bound:g}), rms err/rms = "
              f"{e_rms:.3e}, worst token {int(per_token.argmax())}, tokens over the bound {over.size} of {w.T}, "
              f"oracle {time.time() - t0:.0f} s", flush=True)
        if not fp8:
            assert e <= bound
        else:
            # fp8: the row scale of an activation row is amax / 448.  Where the row's largest bf16
            # activation comes out one ulp (0.8 %) away from the oracle's (float32 against float64
            # accumulation of g and u), every code of that row is taken on a slightly different
            # grid, and with a large combine weight on that row the token leaves the end-to-end
            # bound although every stage is exact (measured: 1.1e-1 on the worst of 32768 tokens).
            # Such tokens must be rare, must pass the stage gates (codes and scales bit-exact on the
            # device's own activations, down projection and combine continued from the device's
            # own codes within 1e-3), and the error over all outputs must stay small.
            assert e_rms <= 5e-3
            assert over.size <= w.T // 1000
            worst = np.argsort(per_token)[-8:]
            import test_gpu_fp8 as tf
            tf._fp8_case(w, np.sort(worst), gate_end_to_end=False)
        del ref, err
