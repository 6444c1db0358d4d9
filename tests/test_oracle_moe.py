"""Pins for the fp64 MoE-block oracle: brute-force loops (Python on a toy, C on
the tiny layer), a case worked by hand, closed forms, invariants, scaling laws
and special cases that collapse to a dense SwiGLU FFN evaluated by torch."""
import math

import numpy as np
import pytest
import torch

import workloads
from oracle import brute, codecs, moe_oracle as mo


def _rand_layer(rng, T, H, E, I, sigma_w=0.3):
    return dict(x=rng.standard_normal((T, H)), w_router=rng.standard_normal((E, H)),
                w_gate=rng.standard_normal((E, I, H)) * sigma_w, w_up=rng.standard_normal((E, I, H)) * sigma_w,
                w_down=rng.standard_normal((E, H, I)) * sigma_w)


def _run(d, k, bias=None, **kw):
    return mo.moe_layer(d["x"], d["w_router"], d["w_gate"], d["w_up"], d["w_down"], k, bias, **kw)


INT_KEYS = ("topk_idx", "counts", "offsets", "perm", "inv_perm")


def test_hand_worked_case():
    """T=1, H=2, E=3, k=2, I=1.  x=(1,2).  Router rows (1,0),(0,1),(1,1) -> logits
    (1,2,3): experts 2 then 1.  w = (e^3, e^2)/(e^3+e^2) = (e, 1)/(e+1).
    Expert e: gate row (1,0)*(e+1) -> g=e+1, up row (0,1) -> u=2, down column (1,-1).
    y_e = silu(e+1)*2*(1,-1);  out = w0*y_2 + w1*y_1."""
    x = np.array([[1.0, 2.0]])
    wr = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    wg = np.array([[[1.0 * (e + 1), 0.0]] for e in range(3)])
    wu = np.array([[[0.0, 1.0]] for _ in range(3)])
    wd = np.array([[[1.0], [-1.0]] for _ in range(3)])
    r = mo.moe_layer(x, wr, wg, wu, wd, 2)
    assert r["topk_idx"].tolist() == [[2, 1]]
    w0 = math.e / (math.e + 1.0)
    assert np.allclose(r["topk_w"], [[w0, 1 - w0]], rtol=0, atol=1e-15)
    s = lambda g: g / (1.0 + math.exp(-g))
    o = w0 * s(3.0) * 2.0 + (1 - w0) * s(2.0) * 2.0
    assert np.allclose(r["out"], [[o, -o]], rtol=1e-15)
    assert r["counts"].tolist() == [0, 1, 1] and r["offsets"].tolist() == [0, 0, 1, 2]
    assert r["perm"].tolist() == [1, 0] and r["inv_perm"].tolist() == [1, 0]


@pytest.mark.parametrize("T,H,E,k,I,with_bias", [(7, 5, 4, 2, 6, False), (5, 8, 6, 3, 4, True), (3, 4, 3, 3, 2, False)])
def test_against_python_loops(T, H, E, k, I, with_bias):
    rng = np.random.default_rng(100 + T)
    d = _rand_layer(rng, T, H, E, I)
    b = rng.standard_normal(E) if with_bias else None
    got = _run(d, k, b)
    ref = brute.moe_layer_loops(d["x"], d["w_router"], d["w_gate"], d["w_up"], d["w_down"], k, b)
    for key in INT_KEYS:
        assert np.array_equal(got[key], ref[key]), key
    assert np.allclose(got["topk_w"], ref["topk_w"], rtol=1e-13, atol=0)
    assert np.allclose(got["out"], ref["out"], rtol=1e-12, atol=1e-13)


def test_against_c_loops_tiny_layer(tiny_inputs):
    d = tiny_inputs
    w = workloads.TINY
    got = _run(d, w.K)
    ref = brute.moe_layer_c(d["x"], d["w_router"], d["w_gate"], d["w_up"], d["w_down"], w.K)
    for key in INT_KEYS:
        assert np.array_equal(got[key], ref[key]), key
    assert np.allclose(got["topk_w"], ref["topk_w"], rtol=1e-12, atol=0)
    rms = np.sqrt(np.mean(ref["out"] ** 2))
    assert np.max(np.abs(got["out"] - ref["out"])) <= 1e-12 * rms


def test_c_loops_match_python_loops():
    rng = np.random.default_rng(9)
    d = _rand_layer(rng, 6, 5, 4, 3)
    b = rng.standard_normal(4)
    a = brute.moe_layer_c(d["x"], d["w_router"], d["w_gate"], d["w_up"], d["w_down"], 2, b)
    p = brute.moe_layer_loops(d["x"], d["w_router"], d["w_gate"], d["w_up"], d["w_down"], 2, b)
    for key in INT_KEYS:
        assert np.array_equal(a[key], p[key]), key
    assert np.allclose(a["out"], p["out"], rtol=1e-13, atol=1e-14)


# ------------------------------------------------------------------ selection
def test_topk_ties_and_special_cases():
    rng = np.random.default_rng(1)
    T, H, E, k = 32, 16, 8, 3
    x = rng.standard_normal((T, H))
    wr = rng.standard_normal((E, H))
    wr[5] = wr[2]                      # experts 2 and 5 always tie
    l = mo.router_logits(x, wr)
    assert np.array_equal(l[:, 2], l[:, 5])
    idx = mo.select_topk(l, k)
    for t in range(T):
        row = list(idx[t])
        if 5 in row:
            assert 2 in row and row.index(2) + 1 == row.index(5)
        vals = l[t, idx[t]]
        assert np.all(np.diff(vals) <= 0)
        assert vals[-1] >= np.delete(l[t], idx[t]).max()
    # all-zero input: every logit equal -> experts 0..k-1, weights 1/k
    z = mo.moe_layer(np.zeros((4, H)), wr, np.zeros((E, 4, H)), np.zeros((E, 4, H)), np.zeros((E, H, 4)), k)
    assert np.array_equal(z["topk_idx"], np.tile(np.arange(k), (4, 1)))
    assert np.array_equal(z["topk_w"], np.full((4, k), 1.0 / k))
    # signed zeros compare equal: lower index first
    assert mo.select_topk(np.array([[0.0, -0.0, 0.0, -1.0]]), 3).tolist() == [[0, 1, 2]]
    assert mo.select_topk(np.array([[-0.0, 0.0, 1.0, 0.0]]), 3).tolist() == [[2, 0, 1]]
    # k = E: a full descending stable sort
    full = mo.select_topk(l, E)
    assert np.array_equal(np.sort(full, axis=1), np.tile(np.arange(E), (T, 1)))
    # one dominant expert takes (almost) all the weight
    l2 = l.copy()
    l2[:, 6] += 60.0
    i2 = mo.select_topk(l2, k)
    w2 = mo.topk_weights(l2, i2)
    assert np.all(i2[:, 0] == 6) and np.all(w2[:, 0] > 1 - 1e-12)


def test_topk_equals_full_sort_bruteforce():
    rng = np.random.default_rng(2)
    l = np.round(rng.standard_normal((200, 17)) * 2) / 2      # many exact ties
    idx = mo.select_topk(l, 5)
    for t in range(l.shape[0]):
        ref = sorted(range(17), key=lambda e: (-l[t, e], e))[:5]
        assert list(idx[t]) == ref


def test_weights_closed_form():
    rng = np.random.default_rng(3)
    l = rng.standard_normal((300, 64)) * 3
    idx = mo.select_topk(l, 8)
    w = mo.topk_weights(l, idx)
    sel = np.take_along_axis(l, idx.astype(np.int64), 1)
    ref = np.exp(sel - sel[:, :1])
    ref /= ref.sum(1, keepdims=True)
    assert np.allclose(w, ref, rtol=1e-13, atol=0)
    assert np.allclose(w.sum(1), 1.0, rtol=0, atol=1e-15)
    assert np.all(np.diff(w, axis=1) <= 0)
    ref_t = torch.softmax(torch.from_numpy(sel), dim=1).numpy()
    assert np.allclose(w, ref_t, rtol=1e-13, atol=0)


def test_logits_linear_and_bias():
    rng = np.random.default_rng(4)
    x = rng.standard_normal((9, 33)).astype(np.float32)
    wr = rng.standard_normal((5, 33)).astype(np.float32)
    b = rng.standard_normal(5).astype(np.float32)
    l = mo.router_logits(x, wr)
    assert np.array_equal(mo.router_logits(4.0 * x, wr), 4.0 * l)
    assert np.array_equal(mo.router_logits(x, wr, b), l + b.astype(np.float64))
    ref = torch.from_numpy(x).double() @ torch.from_numpy(wr).double().T
    assert np.allclose(l, ref.numpy(), rtol=1e-14, atol=1e-14)
    # transposed-operand mistake would not even have this shape / these values
    assert l.shape == (9, 5) and abs(l[2, 3] - float(np.dot(x[2].astype(np.float64), wr[3].astype(np.float64)))) < 1e-13


# ------------------------------------------------------------------ grouping
def test_grouping_invariants():
    rng = np.random.default_rng(6)
    T, E, k = 500, 16, 4
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    idx[:, 0] = np.where(rng.random(T) < 0.7, 3, idx[:, 0])       # skew; may duplicate within a token - allowed here
    counts, offsets, perm, inv = mo.group_by_expert(idx, E)
    flat = idx.reshape(-1)
    assert counts.sum() == T * k and offsets[0] == 0 and offsets[-1] == T * k
    assert np.all(np.diff(offsets) == counts)
    assert np.array_equal(np.sort(perm), np.arange(T * k))
    assert np.array_equal(inv[perm], np.arange(T * k))
    for e in range(E):
        seg = perm[offsets[e]:offsets[e + 1]]
        assert np.all(flat[seg] == e) and np.all(np.diff(seg) > 0)
    # an expert nobody picked
    counts2, offsets2, _, _ = mo.group_by_expert(np.array([[0, 2], [2, 0]]), 4)
    assert counts2.tolist() == [2, 0, 2, 0] and offsets2.tolist() == [0, 2, 2, 4, 4]


# ------------------------------------------------------------------ experts / combine
def _dense_swiglu_torch(x, wg, wu, wd):
    x, wg, wu, wd = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (x, wg, wu, wd))
    return ((torch.nn.functional.silu(x @ wg.T) * (x @ wu.T)) @ wd.T).numpy()


def test_single_expert_is_dense_swiglu():
    rng = np.random.default_rng(7)
    d = _rand_layer(rng, 20, 12, 1, 9)
    r = _run(d, 1)
    assert np.all(r["topk_w"] == 1.0)
    ref = _dense_swiglu_torch(d["x"], d["w_gate"][0], d["w_up"][0], d["w_down"][0])
    assert np.allclose(r["out"], ref, rtol=1e-12, atol=1e-13)


def test_identical_experts_collapse():
    rng = np.random.default_rng(8)
    d = _rand_layer(rng, 40, 10, 6, 7)
    for key in ("w_gate", "w_up", "w_down"):
        d[key] = np.repeat(d[key][:1], 6, axis=0)
    r = _run(d, 3)
    ref = _dense_swiglu_torch(d["x"], d["w_gate"][0], d["w_up"][0], d["w_down"][0])
    assert np.allclose(r["out"], ref, rtol=1e-11, atol=1e-12)


def test_k1_is_unpermute_and_scaling_laws():
    rng = np.random.default_rng(9)
    d = _rand_layer(rng, 30, 8, 5, 6)
    r = _run(d, 1, keep_act=True)
    for t in range(30):
        e = r["topk_idx"][t, 0]
        ref = _dense_swiglu_torch(d["x"][t:t + 1], d["w_gate"][e], d["w_up"][e], d["w_down"][e])
        assert np.allclose(r["out"][t], ref[0], rtol=1e-12, atol=1e-13)
    r3 = _run(d, 3)
    d2 = dict(d, w_down=d["w_down"] * 4.0)
    assert np.array_equal(_run(d2, 3)["out"], r3["out"] * 4.0)
    d3 = dict(d, w_up=np.zeros_like(d["w_up"]))
    assert np.all(_run(d3, 3)["out"] == 0)
    # swapping gate and up must matter (catches crossed operands)
    d4 = dict(d, w_gate=d["w_up"], w_up=d["w_gate"])
    assert not np.allclose(_run(d4, 3)["out"], r3["out"])


def test_token_permutation_and_expert_relabelling():
    rng = np.random.default_rng(10)
    d = _rand_layer(rng, 25, 8, 6, 5)
    r = _run(d, 2)
    p = rng.permutation(25)
    rp = _run(dict(d, x=d["x"][p]), 2)
    assert np.allclose(rp["out"], r["out"][p], rtol=1e-13, atol=1e-14)
    assert np.array_equal(rp["topk_idx"], r["topk_idx"][p])
    q = rng.permutation(6)
    dq = dict(d, w_router=d["w_router"][q], w_gate=d["w_gate"][q], w_up=d["w_up"][q], w_down=d["w_down"][q])
    rq = _run(dq, 2)
    assert np.allclose(rq["out"], r["out"], rtol=1e-12, atol=1e-13)
    assert np.array_equal(q[rq["topk_idx"]], r["topk_idx"])


def test_token_subset_and_device_logit_routing():
    rng = np.random.default_rng(11)
    d = _rand_layer(rng, 50, 8, 6, 5)
    full = _run(d, 2)
    tok = np.array([3, 17, 4, 49])
    sub = _run(d, 2, tokens=tok)
    assert np.allclose(sub["out"], full["out"][tok], rtol=1e-13, atol=1e-14)
    assert np.array_equal(sub["perm"], full["perm"])
    # routing on supplied logits
    l32 = full["logits"].astype(np.float32)
    alt = _run(d, 2, routing_logits=l32)
    assert np.array_equal(alt["topk_idx"], mo.select_topk(l32.astype(np.float64), 2))


# ------------------------------------------------------------------ storage types
def test_bf16_storage_and_act_rounding():
    w = workloads.scaled(workloads.QWEN3_8K, T=64, H=128, E=8, K=2, I=64)
    d = workloads.generate(w)
    assert d["x"].dtype == np.uint16
    pure = _run(d, 2, keep_act=True)
    rp = _run(d, 2, act_rounding="bf16", keep_act=True)
    assert np.array_equal(rp["act"], codecs.f64_to_bf16_value(pure["act"]))
    rms = np.sqrt(np.mean(pure["out"] ** 2))
    gap = np.max(np.abs(rp["out"] - pure["out"])) / rms
    assert 0 < gap < 2e-2
    # stored inputs are used as they are: widening bf16 bits by hand gives the same result
    d32 = {k2: (mo.as_f32(v) if isinstance(v, np.ndarray) and v.dtype == np.uint16 else v) for k2, v in d.items()}
    assert np.array_equal(_run(d32, 2)["out"], pure["out"])


def test_fp8_path_against_torch_casts():
    """Independent fp8 reference: torch's float8_e4m3fn casts for every quantiser,
    float64 matmuls in between."""
    w = workloads.scaled(workloads.QWEN3_32K_FP8, T=48, H=128, E=4, K=2, I=64)
    d = workloads.generate(w)
    r = _run(d, 2, fp8=True, keep_act=True)

    def q_rows(v32):
        v = torch.from_numpy(np.ascontiguousarray(v32, dtype=np.float32))
        amax = v.abs().amax(dim=1)
        s = torch.where(amax == 0, torch.ones_like(amax), amax / 448.0)
        q = (v / s[:, None]).clamp(-448, 448).to(torch.float8_e4m3fn)
        return q.to(torch.float64) * s.to(torch.float64)[:, None]

    x32 = mo.as_f32(d["x"])
    xq = q_rows(x32)
    out = np.zeros((w.T, w.H))
    for t in range(w.T):
        for j in range(2):
            e = int(r["topk_idx"][t, j])
            wg, wu, wd = (q_rows(mo.as_f32(d[n][e])) for n in ("w_gate", "w_up", "w_down"))
            g = xq[t:t + 1] @ wg.T
            u = xq[t:t + 1] @ wu.T
            a = (g / (1 + torch.exp(-g)) * u)
            a_bf = a.to(torch.float32).to(torch.bfloat16).to(torch.float32)   # values far from double-rounding cases are checked below
            aq = q_rows(a_bf.numpy())
            out[t] += r["topk_w"][t, j] * (aq @ wd.T).numpy()[0]
    rms = np.sqrt(np.mean(out ** 2))
    # identical up to rare double-rounding differences of `a` (float64->float32->bf16 in the reference)
    assert np.max(np.abs(r["out"] - out)) <= 2e-3 * rms
    assert np.mean(np.abs(r["out"] - out) > 1e-9 * rms) < 0.02
    # and quantisation matters: the unquantised oracle is far away (so fp8=True is not a no-op)
    pure = _run(d, 2)
    assert np.max(np.abs(r["out"] - pure["out"])) > 5e-2 * rms


def test_down_project_is_the_second_gemm_of_the_layer():
    """down_project referees the down-projection stage of the GPU tests, so it is pinned on its
    own: (1) a case worked by hand; (2) against the y that moe_layer itself returns, for the
    unrounded, the bf16-activation and the fp8 flavours (fp8: fed with the dequantised activation
    codes, as the GPU tests feed it); (3) against plain loops and torch's own e4m3 cast of the
    weights; (4) a wrong expert index, a transposed weight or a skipped dequantisation must fail."""
    # (1) by hand: Wd_1 = [[1,2],[3,4],[5,6]] (H=3, I=2), a = (10, 1) -> y = (12, 34, 56)
    wd = np.zeros((2, 3, 2))
    wd[1] = [[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]]
    assert mo.down_project(np.array([[10.0, 1.0]]), wd, 1).tolist() == [[12.0, 34.0, 56.0]]
    assert mo.down_project(np.array([[10.0, 1.0]]), wd, 0).tolist() == [[0.0, 0.0, 0.0]]
    # (2) the layer's own y, all three flavours
    w = workloads.scaled(workloads.QWEN3_32K_FP8, T=40, H=128, E=5, K=2, I=64)
    d = workloads.generate(w)
    for kw in (dict(), dict(act_rounding="bf16"), dict(fp8=True)):
        r = _run(d, 2, keep_act=True, **kw)
        fp8 = bool(kw.get("fp8"))
        rms = np.sqrt(np.mean(r["y"] ** 2))
        for e in range(w.E):
            t, j = np.nonzero(r["topk_idx"] == e)
            if t.size == 0:
                continue
            a = r["act"][t, j]
            if fp8:     # the layer's down projection reads the per-row e4m3 codes of the bf16 activation
                q, sc = codecs.quantize_rows_e4m3(a.astype(np.float32))
                a = codecs.dequantize_rows_e4m3(q, sc)
            y = mo.down_project(a, d["w_down"], e, fp8=fp8)
            assert np.max(np.abs(y - r["y"][t, j])) <= 1e-13 * rms, (kw, e)
            # (4) planted mistakes are visible at the tolerances the GPU stage checks use (1e-4, 1e-3)
            wrong_e = mo.down_project(a, d["w_down"], (e + 1) % w.E, fp8=fp8)
            assert np.max(np.abs(wrong_e - r["y"][t, j])) > 0.5 * rms
            if fp8:
                no_deq = mo.down_project(a, d["w_down"], e, fp8=False)
                assert np.max(np.abs(no_deq - r["y"][t, j])) > 1e-2 * rms
    # (3) plain loops on the stored bf16 weights, and torch's e4m3 cast for the fp8 weights
    rng = np.random.default_rng(5)
    a = rng.standard_normal((3, w.I))
    e = 3
    wd_e = mo.as_f64(d["w_down"][e])                      # [H, I]
    loops = np.array([[sum(wd_e[h, i] * a[m, i] for i in range(w.I)) for h in range(w.H)] for m in range(3)])
    assert np.allclose(mo.down_project(a, d["w_down"], e), loops, rtol=1e-12, atol=1e-14)
    assert not np.allclose(mo.down_project(a[:, ::-1], d["w_down"], e), loops, rtol=1e-3)
    w32 = torch.from_numpy(mo.as_f32(d["w_down"][e]))
    amax = w32.abs().amax(dim=1)
    s = amax / 448.0
    wq = (w32 / s[:, None]).clamp(-448, 448).to(torch.float8_e4m3fn).to(torch.float64) * s.to(torch.float64)[:, None]
    ref8 = torch.from_numpy(a) @ wq.T
    assert np.allclose(mo.down_project(a, d["w_down"], e, fp8=True), ref8.numpy(), rtol=1e-12, atol=1e-14)


def test_workload_recipe():
    w = workloads.scaled(workloads.QWEN3_64K_ZIPF, T=2048, H=256, I=64)
    d = workloads.generate(w)
    d2 = workloads.generate(w)
    assert all(np.array_equal(d[k2], d2[k2]) for k2 in d if d[k2] is not None)
    assert np.allclose(d["bias"][[0, 1, 127]], [0.0, -1.5 * math.log(2), -1.5 * math.log(128)], rtol=1e-6)
    r = mo.moe_layer(d["x"], d["w_router"], d["w_gate"], d["w_up"], d["w_down"], 8, d["bias"], tokens=np.arange(2))
    c = r["counts"]
    assert c.sum() == 2048 * 8 and c[0] > 20 * max(1, c[100])         # Zipf-like popularity
    xs = mo.as_f64(d["x"])
    assert abs(xs.std() - 1.0) < 0.01 and abs(mo.as_f64(d["w_gate"]).std() - 0.02) < 2e-4
