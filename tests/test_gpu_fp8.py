"""GPU parity of the fp8 (e4m3) expert path, gated stage by stage because a single e4m3 code that
differs on a large activation is visible in the output:
  1. quantiser codes and scales bit-exact against the oracle's float32 quantiser (x rows, weights,
     and the activation rows taken from the device's own bf16 act tap);
  2. gate/up + SwiGLU: act within one bf16 ulp of the oracle's fp8-mode activation;
  3. down projection on the device's own quantised activations against float64: <= 1e-3 * rms;
  4. whole layer against the quantising oracle: max|err| <= 6e-2 * rms(ref)."""
import numpy as np
import pytest
import torch

import paper_2605_02960_amd as moe
import workloads
from oracle import codecs, moe_oracle as mo
import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL_FP8 = 6e-2
TOL_FP8_DOWN = 1e-3     # the fp8 MFMA sums its 64 products per instruction with less than float32 care (measured 2.3-2.7e-4)


def _bf16_dev(a32):
    return torch.from_numpy(np.ascontiguousarray(a32, dtype=np.float32)).to(gu.DEV).to(torch.bfloat16)


def test_quantiser_all_bf16_values_and_scales():
    """Every finite bf16 magnitude, in rows whose largest element sets scales from tiny to huge,
    plus an all-zero row: codes and scales bit-exact against the oracle."""
    bits = np.arange(0x0000, 0x7F80, dtype=np.uint16)                 # all finite non-negative bf16
    vals = codecs.bf16_bits_to_f32(bits)
    rng = np.random.default_rng(0)
    rows = []
    for amax_bits in (0x7F7F, 0x5000, 0x4300, 0x3F80, 0x3F81, 0x3E12, 0x2000, 0x0100, 0x0001):
        amax = codecs.bf16_bits_to_f32(np.array([amax_bits], dtype=np.uint16))[0]
        v = vals[vals <= amax]
        v = v[-4096:] if v.size >= 4096 else np.resize(v, 4096)      # the values nearest amax matter most
        sign = np.where(rng.random(v.size) < 0.5, -1.0, 1.0).astype(np.float32)
        rows.append(v * sign)
        lo = np.resize(vals[vals <= amax][:: max(1, (vals <= amax).sum() // 4095)], 4095)
        rows.append(np.concatenate([lo * sign[:4095], [amax]]).astype(np.float32))
    rows.append(np.zeros(4096, dtype=np.float32))
    a = np.stack(rows).astype(np.float32)
    q, s = moe.moe_quantize_rows_e4m3(_bf16_dev(a))
    torch.cuda.synchronize()
    q_ref, s_ref = codecs.quantize_rows_e4m3(a)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(q.cpu().numpy(), q_ref)


def _quantise_weights(g, cfg):
    out = {}
    for name, rows, cols in (("w_gate", cfg.E * cfg.I, cfg.H), ("w_up", cfg.E * cfg.I, cfg.H),
                             ("w_down", cfg.E * cfg.H, cfg.I)):
        q, s = moe.moe_quantize_rows_e4m3(g[name].reshape(rows, cols))
        out[name] = q
        out["s_" + name[2:]] = s
    return out


def _fp8_case(w, tokens, gate_end_to_end=True):
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    print(f"case {w.name} T={w.T} H={w.H} E={w.E} K={w.K} I={w.I} fp8", flush=True)
    wq = _quantise_weights(g, cfg)
    torch.cuda.synchronize()
    # stage 1a: weight codes and scales against the oracle's quantiser (a few experts)
    for name, shape in (("w_gate", (w.E, w.I, w.H)), ("w_down", (w.E, w.H, w.I))):
        for e in (0, w.E - 1):
            q_ref, s_ref = codecs.quantize_rows_e4m3(mo.as_f32(d[name][e]))
            assert np.array_equal(wq[name].reshape(shape)[e].cpu().numpy(), q_ref)
            assert np.array_equal(wq["s_" + name[2:]].reshape(shape[:2])[e].cpu().numpy(), s_ref)
    g8 = dict(g, w_gate=wq["w_gate"], w_up=wq["w_up"], w_down=wq["w_down"], s_gate=wq["s_gate"],
              s_up=wq["s_up"], s_down=wq["s_down"])
    r = gu.run_staged(cfg, g8)
    info = gu.check_routing_and_grouping(cfg, d, r)
    tok = np.arange(w.T) if tokens is None else tokens
    ref = gu.oracle_out(d, cfg, info["logits_gpu"], tokens=tok, fp8=True, keep_act=True)
    inv = r["inv_perm"].cpu().numpy().reshape(w.T, w.K)[tok].reshape(-1)
    sel = torch.from_numpy(inv).to(gu.DEV).long()
    # stage 2: activations
    act_gpu = r["act"][sel].float().cpu().numpy().astype(np.float64).reshape(len(tok), w.K, w.I)
    diff = np.abs(act_gpu - ref["act"])
    # one bf16 ulp, plus the float32 accumulation noise of the code products (sums of ~1e6 in code
    # units) on activations near zero, where g or u changes sign
    bound = np.abs(ref["act"]) * 2.0 ** -7 * 1.01 + 1e-3 * gu.rms(ref["act"])
    assert np.all(diff <= bound), (
        f"act: max|diff|/rms {diff.max() / gu.rms(ref['act']):.3e}, share over bound {np.mean(diff > bound):.3e}, "
        f"corr {np.corrcoef(act_gpu.ravel(), ref['act'].ravel())[0, 1]:.6f}; worst (gpu, ref): "
        f"{[(float(act_gpu.ravel()[i]), float(ref['act'].ravel()[i])) for i in np.argsort((diff - bound).ravel())[-4:]]}")
    flips = float(np.mean(diff > 0))
    assert flips < 0.05
    # stage 1b: activation codes and scales from the device's own bf16 activations
    q_ref, s_ref = codecs.quantize_rows_e4m3(act_gpu.reshape(-1, w.I).astype(np.float32))
    assert np.array_equal(r["act_q"][sel].cpu().numpy(), q_ref)
    assert np.array_equal(r["act_scale"][sel].cpu().numpy(), s_ref)
    # stage 3: down projection on the device's quantised activations
    a_deq = codecs.dequantize_rows_e4m3(q_ref, s_ref).reshape(len(tok), w.K, w.I)
    idx = r["topk_idx"].cpu().numpy()[tok]
    y_gpu = r["y_perm"][sel].cpu().numpy().reshape(len(tok), w.K, w.H)
    y_ref = np.zeros_like(y_gpu, dtype=np.float64)
    for e in np.unique(idx):
        a_, b_ = np.nonzero(idx == e)
        y_ref[a_, b_] = mo.down_project(a_deq[a_, b_], d["w_down"], e, fp8=True)
    e_down = gu.max_err_over_rms(y_gpu, y_ref)
    # stage 4: whole layer
    out = r["out"].cpu().numpy()[tok]
    e_out = gu.max_err_over_rms(out, ref["out"])
    # stage 4b: the combine of the oracle's down projection on the device's own codes: what the
    # layer must give once the quantisation decisions are taken as the device took them
    out_own = np.einsum("tj,tjh->th", ref["topk_w"][tok], y_ref)
    e_own = gu.max_err_over_rms(out, out_own)
    print(f"  {w.name}: layer max|err|/rms vs quantising oracle {e_out:.3e} (vs the oracle continued from the "
          f"device's own activation codes {e_own:.3e}); down stage {e_down:.3e}; "
          f"bf16 activations differing by one ulp {100 * flips:.4f}%", flush=True)
    assert e_down <= TOL_FP8_DOWN
    assert e_own <= TOL_FP8_DOWN
    # A one-ulp difference of a bf16 activation can flip its e4m3 code (a 6-12 % step of that element);
    # with few terms per output (small I, small K) a handful of flips can move an output past the
    # end-to-end bound although every stage is right, so the bound is asserted at the sizes it is stated for
    # and reported elsewhere.
    if gate_end_to_end:
        assert e_out <= TOL_FP8
    return cfg, g8, r


def test_fp8_small_layer_all_tokens():
    w = workloads.scaled(workloads.QWEN3_32K_FP8, name="fp8_small", T=600, H=256, E=8, K=2, I=512)
    cfg, g8, r = _fp8_case(w, None)
    out = moe.moe_prefill_layer(cfg, g8["x"], g8["w_router"], g8["bias"], g8["w_gate"], g8["w_up"], g8["w_down"],
                                g8["s_gate"], g8["s_up"], g8["s_down"])
    torch.cuda.synchronize()
    assert torch.equal(out, r["out"])


def test_fp8_qwen3_layer_32k_tokens():
    w = workloads.QWEN3_32K_FP8
    tokens = np.sort(np.random.default_rng(3).choice(w.T, size=128, replace=False))
    cfg, g8, r = _fp8_case(w, tokens)
    # the call as bench.py makes it (fused, no taps) gives the same bits as the staged calls
    out = moe.moe_prefill_layer(cfg, g8["x"], g8["w_router"], g8["bias"], g8["w_gate"], g8["w_up"], g8["w_down"],
                                g8["s_gate"], g8["s_up"], g8["s_down"])
    torch.cuda.synchronize()
    assert torch.equal(out, r["out"])


@pytest.mark.parametrize("T,E,K,zipf", [(96, 8, 2, False), (96, 8, 8, False), (128, 12, 4, True)],
                         ids=["k2", "k_eq_e", "zipf"])
def test_fp8_full_contraction_lengths_all_tokens(T, E, K, zipf):
    """The real contraction lengths of the fp8 configuration (H = 4096, I = 1536) on a batch small
    enough for the oracle to evaluate every token: every stage gate, and the end-to-end bound of
    6e-2 * rms asserted over all tokens."""
    w = workloads.scaled(workloads.QWEN3_32K_FP8, name=f"fp8_full_hi_{T}_{E}_{K}_{int(zipf)}", T=T, E=E, K=K,
                         zipf_bias=zipf)
    cfg, g8, r = _fp8_case(w, None, gate_end_to_end=True)
    out = moe.moe_prefill_layer(cfg, g8["x"], g8["w_router"], g8["bias"], g8["w_gate"], g8["w_up"], g8["w_down"],
                                g8["s_gate"], g8["s_up"], g8["s_down"])
    torch.cuda.synchronize()
    assert torch.equal(out, r["out"])


@pytest.mark.parametrize("T,H,E,K,I", [
    (1, 256, 3, 3, 256),       # one token, every expert chosen
    (130, 256, 1, 1, 512),     # one expert, a group that ends two rows into a 64-row block
    (40, 256, 1024, 32, 256),  # the largest expert count and the largest K: mostly empty and one-row groups
], ids=["one_token_k_eq_e", "one_expert", "e1024_k32"])
def test_fp8_degenerate_shapes(T, H, E, K, I):
    w = workloads.scaled(workloads.QWEN3_32K_FP8, name=f"fp8_degenerate_{T}_{H}_{E}_{K}_{I}", T=T, H=H, E=E, K=K, I=I)
    cfg, g8, r = _fp8_case(w, None, gate_end_to_end=False)
    out = moe.moe_prefill_layer(cfg, g8["x"], g8["w_router"], g8["bias"], g8["w_gate"], g8["w_up"], g8["w_down"],
                                g8["s_gate"], g8["s_up"], g8["s_down"])
    torch.cuda.synchronize()
    assert torch.equal(out, r["out"])


@pytest.mark.parametrize("seed", range(5))
def test_fp8_random_small_shapes(seed):
    """Seeded random shapes of the fp8 path (H, I multiples of 256; any T, E, K; with and without
    the skewing router bias): every stage and every token against the quantising oracle, fused ==
    staged."""
    rng = np.random.default_rng(2000 + seed)
    H, I = 256 * int(rng.integers(1, 3)), 256 * int(rng.integers(1, 3))
    E = int(rng.integers(1, 25))
    K = int(rng.integers(1, min(E, 8) + 1))
    T = int(rng.integers(1, 900))
    w = workloads.scaled(workloads.QWEN3_32K_FP8, name=f"fp8_rand{seed}_{T}_{H}_{E}_{K}_{I}", T=T, H=H, E=E, K=K, I=I,
                         zipf_bias=bool(rng.integers(0, 2)))
    cfg, g8, r = _fp8_case(w, None, gate_end_to_end=False)
    out = moe.moe_prefill_layer(cfg, g8["x"], g8["w_router"], g8["bias"], g8["w_gate"], g8["w_up"], g8["w_down"],
                                g8["s_gate"], g8["s_up"], g8["s_down"])
    torch.cuda.synchronize()
    assert torch.equal(out, r["out"])
