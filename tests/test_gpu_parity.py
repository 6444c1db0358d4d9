"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer outputs (routing, grouping) must be bit-exact against the oracle's
selection on the device's own float32 logits; floating-point outputs within the stated bounds:
  float32 configuration : max|err| <= 1e-4 * rms(ref)
  bf16                  : max|err| <= 2e-2 * rms(ref) on the float32 result against the oracle
                          without intermediate rounding, and <= 5e-3 * rms(ref) against the oracle
                          that rounds the SwiGLU activation to bf16 as the bf16 model does
"""
import numpy as np
import pytest
import torch

import paper_2605_02960_amd as moe
import workloads
from oracle import codecs, moe_oracle as mo
import gpu_util as gu
import y_block16 as yb

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4
TOL_BF16_PURE = 2e-2
TOL_BF16_RP = 5e-3       # dominated by rare one-ulp differences of single bf16 activations
TOL_DOWN_STAGE = 1e-4    # float32 accumulation of exact bf16 products over I terms


def _fused(cfg, g, taps=None):
    out = moe.moe_prefill_layer(cfg, g["x"], g["w_router"], g["bias"], g["w_gate"], g["w_up"], g["w_down"],
                                g.get("s_gate"), g.get("s_up"), g.get("s_down"), taps=taps)
    torch.cuda.synchronize()
    return out


def _layer_case(w, tokens=None, seed=0):
    d = workloads.generate(w, seed=seed)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    print(f"case {w.name} T={w.T} H={w.H} E={w.E} K={w.K} I={w.I} {w.dtype}", flush=True)
    r = gu.run_staged(cfg, g)
    info = gu.check_routing_and_grouping(cfg, d, r)
    return d, g, cfg, r, info


# ------------------------------------------------------------------ float32 configuration
def test_tiny_fp32_layer():
    w = workloads.TINY
    d, g, cfg, r, info = _layer_case(w)
    pure = gu.oracle_out(d, cfg, info["logits_gpu"], keep_act=True)
    # act tap: rows in sorted order
    perm = pure["perm"]
    act_ref = pure["act"].reshape(w.T * w.K, w.I)[perm]
    assert gu.max_err_over_rms(r["act"].cpu().numpy(), act_ref) <= TOL_F32
    y_ref = pure["y"].reshape(w.T * w.K, w.H)[perm]
    assert gu.max_err_over_rms(r["y_perm"].cpu().numpy(), y_ref) <= TOL_F32
    assert gu.max_err_over_rms(r["out"].cpu().numpy(), pure["out"]) <= TOL_F32
    assert info["same_set_as_f64"] == 1.0
    # fused call == staged calls, bitwise
    assert torch.equal(_fused(cfg, g), r["out"])


@pytest.mark.parametrize("T,H,E,K,I,zipf", [
    (37, 50, 5, 3, 33, False),      # nothing divides anything
    (1, 7, 3, 1, 5, False),
    (300, 96, 70, 7, 40, True),     # E > 64: two logits per lane; skewed groups
    (129, 64, 1024, 32, 16, False), # the limits of E and K
    (64, 32, 6, 6, 24, False),      # K = E
])
def test_fp32_ragged_shapes(T, H, E, K, I, zipf):
    w = workloads.scaled(workloads.TINY, name=f"f32_{T}_{H}_{E}_{K}_{I}", T=T, H=H, E=E, K=K, I=I, zipf_bias=zipf)
    d, g, cfg, r, info = _layer_case(w)
    pure = gu.oracle_out(d, cfg, info["logits_gpu"])
    assert gu.max_err_over_rms(r["out"].cpu().numpy(), pure["out"]) <= TOL_F32
    assert torch.equal(_fused(cfg, g), r["out"])


def test_empty_batch():
    w = workloads.scaled(workloads.TINY, T=0)
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    r = gu.run_staged(cfg, g)
    assert r["out"].shape == (0, w.H)
    assert r["counts"].cpu().tolist() == [0] * w.E and r["offsets"].cpu().tolist() == [0] * (w.E + 1)
    assert _fused(cfg, g).shape == (0, w.H)


def test_ties_zero_input_and_dominant_expert():
    w = workloads.scaled(workloads.TINY, T=96, E=8, K=3)
    d = workloads.generate(w)
    d["w_router"][5] = d["w_router"][2]          # experts 2 and 5 tie on every token
    d["x"][:16] = 0.0                            # all logits equal: experts 0..K-1, weights 1/K
    d["w_router"][7] *= 400.0                    # a dominant (positive or negative) expert
    g = gu.upload(d)
    cfg = gu.config_for(w)
    r = gu.run_staged(cfg, g)
    info = gu.check_routing_and_grouping(cfg, d, r)
    idx = r["topk_idx"].cpu().numpy()
    wt = r["topk_w"].cpu().numpy()
    assert np.array_equal(idx[:16], np.tile(np.arange(3), (16, 1)))
    assert np.array_equal(wt[:16], np.full((16, 3), np.float32(1.0) / np.float32(3.0)))
    for t in range(16, 96):
        row = list(idx[t])
        if 5 in row:
            assert 2 in row and row.index(2) + 1 == row.index(5)
    pure = gu.oracle_out(d, cfg, info["logits_gpu"])
    assert gu.max_err_over_rms(r["out"].cpu().numpy(), pure["out"]) <= TOL_F32


def test_identical_experts_collapse_to_dense_ffn():
    """With identical experts the block is a dense SwiGLU FFN whatever the routing."""
    w = workloads.scaled(workloads.TINY, T=80, E=6, K=3)
    d = workloads.generate(w)
    for k in ("w_gate", "w_up", "w_down"):
        d[k][:] = d[k][0]
    g = gu.upload(d)
    cfg = gu.config_for(w)
    r = gu.run_staged(cfg, g)
    x = d["x"].astype(np.float64)
    gte = x @ d["w_gate"][0].astype(np.float64).T
    ref = (gte / (1 + np.exp(-gte)) * (x @ d["w_up"][0].astype(np.float64).T)) @ d["w_down"][0].astype(np.float64).T
    assert gu.max_err_over_rms(r["out"].cpu().numpy(), ref) <= TOL_F32


def test_permute_with_gather_and_k1_unpermute():
    w = workloads.scaled(workloads.TINY, T=200, E=8, K=1)
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    idx, wt, _ = moe.moe_route(cfg, g["x"], g["w_router"], None)
    counts, offsets, perm, inv, xp = moe.moe_permute(cfg, idx, g["x"], want_x_perm=True)
    torch.cuda.synchronize()
    assert torch.equal(xp, g["x"][(perm // cfg.K).long()])
    assert torch.all(wt == 1.0)
    # K = 1: combine is a pure un-permute
    y = torch.randn((w.T, w.H), device=gu.DEV)
    out = moe.moe_combine(cfg, y, inv, wt)
    assert torch.equal(out, y[inv.long()])


# ------------------------------------------------------------------ bf16 (MFMA path)
def _bf16_checks(w, d, g, cfg, r, info, tokens):
    pure = gu.oracle_out(d, cfg, info["logits_gpu"], tokens=tokens)
    rp = gu.oracle_out(d, cfg, info["logits_gpu"], tokens=tokens, act_rounding="bf16", keep_act=True)
    out = r["out"].cpu().numpy()[pure["tokens"]]
    e_pure = gu.max_err_over_rms(out, pure["out"])
    e_rp = gu.max_err_over_rms(out, rp["out"])
    floor = gu.max_err_over_rms(rp["out"], pure["out"])
    print(f"  {w.name}: max|err|/rms vs unrounded oracle {e_pure:.3e} (rounding floor {floor:.3e}), "
          f"vs bf16-activation oracle {e_rp:.3e}; same expert set as float64 routing "
          f"{100 * info['same_set_as_f64']:.3f}%", flush=True)
    assert e_rp <= TOL_BF16_RP
    assert e_pure <= TOL_BF16_PURE
    # Stage 1, act tap (bf16): the oracle's bf16-rounded activation, up to one bf16 ulp where the
    # float32 accumulation error moves a value across a rounding boundary, plus that accumulation
    # error itself on values near zero (g or u close to a sign change).
    inv = r["inv_perm"].cpu().numpy().reshape(w.T, w.K)[pure["tokens"]]          # sorted positions
    act_gpu = r["act"].float().cpu().numpy().astype(np.float64)[inv.reshape(-1)]
    act_gpu = act_gpu.reshape(len(pure["tokens"]), w.K, w.I)
    diff = np.abs(act_gpu - rp["act"])
    ulp = np.abs(rp["act"]) * 2.0 ** -7
    assert np.all(diff <= ulp * 1.01 + 1e-4 * gu.rms(rp["act"]))
    assert np.mean(diff > 0) < 0.02
    # Stage 2, down projection on the device's own bf16 activations: float32 accumulation only.
    idx = r["topk_idx"].cpu().numpy()[pure["tokens"]]
    y_gpu = r["y_perm"][torch.from_numpy(inv.reshape(-1)).to(gu.DEV).long()].cpu().numpy()
    y_gpu = y_gpu.reshape(len(pure["tokens"]), w.K, w.H)
    y_ref = np.zeros_like(y_gpu, dtype=np.float64)
    for e in np.unique(idx):
        a_, b_ = np.nonzero(idx == e)
        y_ref[a_, b_] = mo.down_project(act_gpu[a_, b_], d["w_down"], e)
    e_down = gu.max_err_over_rms(y_gpu, y_ref)
    print(f"  down projection on the device's activations: max|err|/rms {e_down:.3e}; "
          f"activation elements that differ from the oracle's by one bf16 ulp: {100 * np.mean(diff > 0):.4f}%", flush=True)
    # y is handed over in block-scaled 16-bit form unless the configuration keeps float32: at most
    # half a code step of the element's block on top of the float32 accumulation error
    step = 0.0 if (cfg.flags & moe.FLAG_Y_F32) else gu.block16_half_step(y_ref) * 1.02 + 2e-5 * gu.rms(y_ref)
    assert np.all(np.abs(y_gpu - y_ref) <= step + TOL_DOWN_STAGE * gu.rms(y_ref))
    return pure, rp


def test_bf16_small_skewed_with_empty_experts():
    w = workloads.scaled(workloads.QWEN3_64K_ZIPF, name="bf16_small_zipf", T=700, H=256, E=32, K=4, I=384)
    d, g, cfg, r, info = _layer_case(w)
    assert int((r["counts"] == 0).sum()) >= 1       # the Zipf-like bias leaves the rarest experts without rows
    _bf16_checks(w, d, g, cfg, r, info, None)
    assert torch.equal(_fused(cfg, g), r["out"])
    # determinism: a second run is bitwise identical
    r2 = gu.run_staged(cfg, g)
    assert torch.equal(r2["out"], r["out"]) and torch.equal(r2["y_perm"], r["y_perm"])


def test_bf16_router_ragged_expert_and_token_tiles():
    """E = 160 (one full and one partial 128-expert tile), T = 300 (partial 128-token tiles), with a
    router bias: the matrix-core router against the float64 logits, selection bit-exact."""
    w = workloads.scaled(workloads.QWEN3_64K_ZIPF, name="bf16_router_ragged", T=300, H=384, E=160, K=6, I=128)
    d, g, cfg, r, info = _layer_case(w)
    l_ref = mo.router_logits(d["x"], d["w_router"], d["bias"])
    assert gu.max_err_over_rms(r["logits"].cpu().numpy(), l_ref) <= 2e-6     # float32 accumulation of exact products
    _bf16_checks(w, d, g, cfg, r, info, None)
    # want_logits=False: logits live in the workspace, same routing
    idx2, w2, _ = moe.moe_route(cfg, g["x"], g["w_router"], g["bias"], want_logits=False)
    torch.cuda.synchronize()
    assert torch.equal(idx2, r["topk_idx"]) and torch.equal(w2, r["topk_w"])


def test_bf16_group_sizes_around_tile_edges():
    """Groups of 0, 1, 255, 256, 257 and 600 rows (K=1, routing forced by the router bias)."""
    sizes = [0, 1, 255, 256, 257, 600, 0, 3]
    T = sum(sizes)
    w = workloads.scaled(workloads.QWEN3_8K, name="bf16_tile_edges", T=T, H=128, E=len(sizes), K=1, I=128)
    d = workloads.generate(w)
    # force token t to expert e(t): a one-hot pattern planted in the first E features
    owner = np.repeat(np.arange(len(sizes)), sizes)
    rng = np.random.default_rng(0)
    owner = owner[rng.permutation(T)]
    x = codecs.bf16_bits_to_f32(d["x"]).copy()
    x[:, :w.E] = 0.0
    x[np.arange(T), owner] = 64.0
    d["x"] = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    d["w_router"][:] = 0.0
    d["w_router"][np.arange(w.E), np.arange(w.E)] = 1.0
    g = gu.upload(d)
    cfg = gu.config_for(w)
    r = gu.run_staged(cfg, g)
    info = gu.check_routing_and_grouping(cfg, d, r)
    assert r["counts"].cpu().tolist() == sizes
    _bf16_checks(w, d, g, cfg, r, info, None)


@pytest.mark.parametrize("T,H,E,K,I,flags", [
    (700, 1024, 6, 2, 1152, 0),                  # 16 and 18 K steps per tile: both GEMMs on 16 x 16 x 32 blocks
    (523, 1152, 5, 3, 1024, moe.FLAG_Y_F32),     # same, float32 y
    (300, 1024, 3, 1, 896, 0),                   # gate/up on 16 x 16 blocks, down (14 K steps) on 32 x 32
], ids=["blk16_both", "blk16_both_yf32", "blk16_gate_up_only"])
def test_bf16_long_contraction_small_batch(T, H, E, K, I, flags):
    """Contractions long enough for the kernels to choose 16 x 16 x 32 MFMA blocks (16 or more K
    steps of 64 per tile), at a size where every token is checked against the oracle: ragged
    groups, tiles with one to three row blocks, both storage forms of y, fused == staged."""
    w = workloads.scaled(workloads.QWEN3_64K_ZIPF, name=f"bf16_longk_{T}_{H}_{E}_{K}_{I}_{flags}", T=T, H=H, E=E, K=K, I=I)
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w, flags=flags)
    print(f"case {w.name} flags={flags}", flush=True)
    r = gu.run_staged(cfg, g)
    info = gu.check_routing_and_grouping(cfg, d, r)
    _bf16_checks(w, d, g, cfg, r, info, None)
    assert torch.equal(_fused(cfg, g), r["out"])


def test_bf16_out_is_rounded_f32_out():
    w = workloads.scaled(workloads.QWEN3_8K, name="bf16_out", T=300, H=256, E=16, K=4, I=128)
    d = workloads.generate(w)
    g = gu.upload(d)
    o32 = _fused(gu.config_for(w), g)
    o16 = _fused(gu.config_for(w, moe.DTYPE_BF16), g)
    assert o16.dtype == torch.bfloat16
    assert torch.equal(o16, o32.to(torch.bfloat16))


def test_bf16_token_permutation_equivariance():
    w = workloads.scaled(workloads.QWEN3_8K, name="bf16_equiv", T=512, H=256, E=16, K=4, I=128)
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    o = _fused(cfg, g)
    p = torch.randperm(w.T, device=gu.DEV, generator=torch.Generator(device=gu.DEV).manual_seed(1))
    g2 = dict(g, x=g["x"][p].contiguous())
    assert torch.equal(_fused(cfg, g2), o[p])


def test_qwen3_layer_8k_tokens():
    """The 235B-A22B-shaped layer at T=8192 (uniform-ish routing): all integer outputs checked in
    full, floating-point outputs on a sample of tokens the oracle evaluates one by one."""
    w = workloads.QWEN3_8K
    d, g, cfg, r, info = _layer_case(w)
    tokens = np.random.default_rng(1).choice(w.T, size=192, replace=False)
    _bf16_checks(w, d, g, cfg, r, info, np.sort(tokens))
    assert info["same_set_as_f64"] > 0.999
    assert torch.equal(_fused(cfg, g), r["out"])


@pytest.mark.parametrize("w", [workloads.QWEN3_64K_ZIPF, workloads.QWEN3_30B_64K_ZIPF], ids=lambda w: w.name)
def test_full_size_layer_64k_tokens_zipf(w):
    """Full size of the bench workloads (T=65536, Zipf-like expert popularity; the 235B-A22B
    layer shape and the 30B-A3B one), same launch configuration as bench.py: integer outputs in
    full, sampled tokens for the floats, plus properties that hold at any size."""
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    print(f"case {w.name}", flush=True)
    taps = dict(logits=torch.empty((w.T, w.E), dtype=torch.float32, device=gu.DEV),
                topk_idx=torch.empty((w.T, w.K), dtype=torch.int32, device=gu.DEV),
                topk_w=torch.empty((w.T, w.K), dtype=torch.float32, device=gu.DEV),
                counts=torch.empty((w.E,), dtype=torch.int32, device=gu.DEV),
                offsets=torch.empty((w.E + 1,), dtype=torch.int32, device=gu.DEV),
                perm=torch.empty((w.rows,), dtype=torch.int32, device=gu.DEV),
                inv_perm=torch.empty((w.rows,), dtype=torch.int32, device=gu.DEV),
                act=torch.empty((w.rows, w.I), dtype=torch.bfloat16, device=gu.DEV),
                y_perm=torch.empty((w.rows, w.H), dtype=torch.float32, device=gu.DEV))
    out = _fused(cfg, g, taps)
    r = dict(taps, out=out)
    info = gu.check_routing_and_grouping(cfg, d, r)
    c = r["counts"].cpu().numpy()
    assert c.sum() == w.rows and c[0] > 50 * max(1, c[-1])
    rng = np.random.default_rng(2)
    # tokens from the crowded head experts and from the rarest experts' groups
    perm = r["perm"].cpu().numpy()
    off = r["offsets"].cpu().numpy()
    rare = perm[off[96]:off[128]] // w.K
    tokens = np.unique(np.concatenate([rng.choice(w.T, size=2048, replace=False), rare[:64]]))
    _bf16_checks(w, d, g, cfg, r, info, tokens)
    assert torch.isfinite(out).all()
    # the call as bench.py makes it (no taps: y stays in its compact form) gives the same bits
    del taps, r
    assert torch.equal(_fused(cfg, g), out)


def test_bf16_layer_with_more_than_4gib_of_activations():
    """T = 196608 tokens at the 235B-A22B layer shape: 1.57 M routed rows, so the bf16 activation
    matrix (4.8 GB) cannot be addressed with 32-bit byte offsets from its start.  Integer outputs
    in full; floats on sampled tokens, among them tokens whose rows sit past the 4 GiB mark."""
    w = workloads.scaled(workloads.QWEN3_8K, name="qwen3_235b_T196608_bf16", T=196608)
    assert w.rows * w.I * 2 > 2 ** 32
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    print(f"case {w.name}", flush=True)
    taps = dict(logits=torch.empty((w.T, w.E), dtype=torch.float32, device=gu.DEV),
                topk_idx=torch.empty((w.T, w.K), dtype=torch.int32, device=gu.DEV),
                topk_w=torch.empty((w.T, w.K), dtype=torch.float32, device=gu.DEV),
                counts=torch.empty((w.E,), dtype=torch.int32, device=gu.DEV),
                offsets=torch.empty((w.E + 1,), dtype=torch.int32, device=gu.DEV),
                perm=torch.empty((w.rows,), dtype=torch.int32, device=gu.DEV),
                inv_perm=torch.empty((w.rows,), dtype=torch.int32, device=gu.DEV),
                act=torch.empty((w.rows, w.I), dtype=torch.bfloat16, device=gu.DEV),
                y_perm=torch.empty((w.rows, w.H), dtype=torch.float32, device=gu.DEV))
    out = _fused(cfg, g, taps)
    r = dict(taps, out=out)
    info = gu.check_routing_and_grouping(cfg, d, r)
    perm = r["perm"].cpu().numpy()
    first_high = (2 ** 32) // (w.I * 2) + 1                   # first sorted row past 4 GiB
    high = perm[first_high::4099][:96] // w.K
    rng = np.random.default_rng(3)
    tokens = np.unique(np.concatenate([rng.choice(w.T, size=160, replace=False), high]))
    _bf16_checks(w, d, g, cfg, r, info, tokens)
    assert torch.isfinite(out).all()
    # the call as bench.py makes it (no taps: y stays in its compact form) gives the same bits
    del taps, r
    assert torch.equal(_fused(cfg, g), out)


def test_y_block16_storage_is_the_quantiser_applied_to_the_float32_result():
    """The down projection's float32 accumulators (MOE_FLAG_Y_F32) against the oracle as before;
    the default block-scaled 16-bit y, seen through the float32 tap, is bit for bit the library's
    quantiser (restated in tests/y_block16.py) applied to those accumulators; and the fused call,
    which keeps y in the compact form, gives the same output bits as the staged calls."""
    w = workloads.scaled(workloads.QWEN3_64K_ZIPF, name="bf16_y_storage", T=900, H=384, E=16, K=4, I=256)
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg16, cfg32 = gu.config_for(w), gu.config_for(w, flags=moe.FLAG_Y_F32)
    r16, r32 = gu.run_staged(cfg16, g), gu.run_staged(cfg32, g)
    assert torch.equal(r16["act"], r32["act"]) and torch.equal(r16["perm"], r32["perm"])
    y32 = r32["y_perm"].cpu().numpy()
    codes, k = yb.quantize_blocks_i16(y32)
    want = yb.dequantize_blocks_i16(codes, k)
    got = r16["y_perm"].cpu().numpy()
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert np.all(np.abs(got - y32) <= gu.block16_half_step(y32.astype(np.float64)))
    assert np.abs(codes).max() > 16000 and k.min() >= 15
    # float32 y: the stage-wise bound without the storage term
    info = gu.check_routing_and_grouping(cfg32, d, r32)
    _bf16_checks(w, d, g, cfg32, r32, info, None)
    assert torch.equal(_fused(cfg32, g), r32["out"])
    # default: compact y inside the fused call == float32 copy of the same values in the staged calls
    assert torch.equal(_fused(cfg16, g), r16["out"])
    assert gu.max_err_over_rms(r16["out"].cpu().numpy(), r32["out"].cpu().numpy()) <= 3e-4


@pytest.mark.parametrize("T,H,E,K,I", [
    (1, 128, 4, 4, 128),       # one token, every expert chosen (K = E): four groups of one row
    (1, 256, 1, 1, 128),       # one token, one expert
    (300, 128, 1, 1, 256),     # one expert takes everything: a single group of two row tiles
    (65, 384, 7, 7, 128),      # K = E: every group has all T rows (one row past a 64-row block)
], ids=["one_token_k_eq_e", "one_token_one_expert", "one_expert", "k_eq_e"])
def test_bf16_degenerate_shapes(T, H, E, K, I):
    """The smallest and the most lopsided cases the method has, every token checked."""
    w = workloads.scaled(workloads.QWEN3_64K_ZIPF, name=f"bf16_degenerate_{T}_{H}_{E}_{K}_{I}", T=T, H=H, E=E, K=K, I=I)
    d, g, cfg, r, info = _layer_case(w)
    assert int(r["counts"].sum()) == T * K
    _bf16_checks(w, d, g, cfg, r, info, None)
    assert torch.equal(_fused(cfg, g), r["out"])


@pytest.mark.parametrize("T,H,E,K,I,dtype", [
    (70, 128, 128, 32, 128, "bf16"),     # selection inside the router kernel, both halves of its 2 x 16 result slots
    (70, 128, 40, 32, 128, "bf16"),      # the same with a ragged expert count
    (70, 128, 256, 32, 128, "bf16"),     # two expert tiles: router GEMM and selection kernel
    (70, 128, 1024, 32, 128, "bf16"),    # the largest expert count the configuration allows
    (50, 64, 64, 32, 64, "fp32"),        # float32 path
], ids=["e128", "e40", "e256", "e1024", "f32_e64"])
def test_largest_k(T, H, E, K, I, dtype):
    """K = 32, the largest the configuration allows: routing bit-exact, weights within 1e-6, layer
    output within the configuration's bound, fused == staged."""
    base = workloads.TINY if dtype == "fp32" else workloads.QWEN3_8K
    w = workloads.scaled(base, name=f"kmax_{dtype}_{E}", T=T, H=H, E=E, K=K, I=I)
    d, g, cfg, r, info = _layer_case(w)
    assert int(r["counts"].sum()) == T * K
    if dtype == "fp32":
        pure = gu.oracle_out(d, cfg, info["logits_gpu"])
        assert gu.max_err_over_rms(r["out"].cpu().numpy(), pure["out"]) <= TOL_F32
    else:
        _bf16_checks(w, d, g, cfg, r, info, None)
    assert torch.equal(_fused(cfg, g), r["out"])


def _random_bf16_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    H = 128 * int(rng.integers(1, 5))
    I = 128 * int(rng.integers(1, 5))
    E = int(rng.integers(1, 41))
    K = int(rng.integers(1, min(E, 9) + 1))
    T = int(rng.integers(1, 1400))
    return T, H, E, K, I, bool(rng.integers(0, 2))


@pytest.mark.parametrize("seed", range(8))
def test_bf16_random_small_shapes(seed):
    """Seeded random shapes of the bf16 path (H, I multiples of 128; any T, E, K): every token
    against the oracle, fused == staged, both storage forms of y."""
    T, H, E, K, I, zipf = _random_bf16_shape(seed)
    w = workloads.scaled(workloads.QWEN3_64K_ZIPF, name=f"bf16_rand{seed}_{T}_{H}_{E}_{K}_{I}", T=T, H=H, E=E, K=K, I=I,
                         zipf_bias=zipf)
    d, g, cfg, r, info = _layer_case(w)
    _bf16_checks(w, d, g, cfg, r, info, None)
    assert torch.equal(_fused(cfg, g), r["out"])
    cfg32 = gu.config_for(w, flags=moe.FLAG_Y_F32)
    o32 = _fused(cfg32, g)
    assert gu.max_err_over_rms(r["out"].cpu().numpy(), o32.cpu().numpy()) <= 5e-4


def test_fused_call_can_be_captured_in_a_graph():
    """The library enqueues kernels only (no allocation, no host synchronisation, no memset node),
    so a caller may capture the fused call in a HIP graph: three replays, with eager work on the
    same buffers in between, each equal to the eager result bit for bit."""
    w = workloads.scaled(workloads.QWEN3_64K_ZIPF, name="bf16_graph", T=1000, H=256, E=24, K=4, I=384)
    d = workloads.generate(w)
    g = gu.upload(d)
    cfg = gu.config_for(w)
    ws = torch.empty(moe.moe_workspace_bytes(cfg, moe.CALL_PREFILL_LAYER), dtype=torch.uint8, device=gu.DEV)
    args = (cfg, g["x"], g["w_router"], g["bias"], g["w_gate"], g["w_up"], g["w_down"])
    want = moe.moe_prefill_layer(*args, ws=ws).clone()         # also the first call: kernel attributes are set here
    torch.cuda.synchronize()
    out = torch.empty_like(want)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        moe.moe_prefill_layer(*args, out=out, ws=ws)
    for rep in range(3):
        out.fill_(float("nan"))
        ws.random_(0, 255)                                      # scratch contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), rep
        eager = moe.moe_prefill_layer(*args, ws=ws)             # the program's own eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(eager, want)
