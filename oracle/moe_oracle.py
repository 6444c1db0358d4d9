"""fp64 oracle of the per-layer MoE block (test infrastructure only).

What the block is (Sec. 2.3 of the paper): the FFN of a decoder block is
replaced by E experts, each a two-layer MLP; a router dispatches every token to
its top-k experts and the k expert outputs are summed.  In the paper's backend
(Sec. 6.2) every GPU holds the whole expert set of the current layer, so the
dispatch is local: this file is that local block and nothing else.

The paper fixes no more than that.  The concrete form used here (softmax
router, selection on the logits, weights renormalised over the selected k,
SwiGLU experts without biases) is the reading listed in the design notes:

  logits   l[t,e] = sum_h x[t,h] * Wr[e,h] (+ b[e])
  select   the k largest l[t,:], listed by descending value; equal values are
           ordered by ascending expert index
  weights  p = softmax(l[t,:]) over all E;  w_j = p[idx_j] / sum_{i<k} p[idx_i]
  group    stable sort of the T*k (token,slot) pairs by expert id
  expert   g = Wg_e x, u = Wu_e x, a = g/(1+exp(-g)) * u, y = Wd_e a
  combine  out[t] = sum_j w_j * y[t,j]

All arithmetic is float64 on the stored input values.  Two optional rounding
points mirror what a bf16 / fp8 model holds in memory between the two expert
GEMMs (they are part of the method's data types, not of any kernel):
  act_rounding="bf16"  a is rounded once to bf16 before the down projection
  fp8=True             expert weights are e4m3 with one float32 scale per output
                       channel; x rows and (bf16-rounded) a rows are quantised
                       per row to e4m3 with a float32 scale; products are then
                       exact float64 on the dequantised values
"""
import numpy as np

from . import codecs


def as_f64(a):
    """Stored tensor -> float64.  uint16 arrays are bf16 bit patterns."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return codecs.bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def as_f32(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return codecs.bf16_bits_to_f32(a)
    return a.astype(np.float32)


# ------------------------------------------------------------------ routing
def router_logits(x, w_router, bias=None):
    """l[t,e] = <x[t,:], Wr[e,:]> (+ b[e]) in float64."""
    l = as_f64(x) @ as_f64(w_router).T
    if bias is not None:
        l = l + as_f64(bias)[None, :]
    return l


def select_topk(logits, k):
    """Indices [T,k] of the k largest logits per row, in descending order of
    value; among equal values the lower expert index comes first (-0.0 == +0.0)."""
    logits = np.asarray(logits, dtype=np.float64)
    order = np.argsort(-logits, axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def topk_weights(logits, idx):
    """Softmax over all E, taken at the selected experts, renormalised to sum 1."""
    logits = np.asarray(logits, dtype=np.float64)
    m = logits.max(axis=1, keepdims=True)
    p = np.exp(logits - m)
    p = p / p.sum(axis=1, keepdims=True)
    sel = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    return sel / sel.sum(axis=1, keepdims=True)


# ------------------------------------------------------------------ grouping
def group_by_expert(topk_idx, E):
    """counts[E], offsets[E+1] (exclusive scan), perm[T*k] (sorted row -> flat id
    t*k+j, ordered by expert then by flat id), inv_perm[T*k] (its inverse)."""
    flat = np.asarray(topk_idx, dtype=np.int64).reshape(-1)
    counts = np.bincount(flat, minlength=E).astype(np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    perm = np.argsort(flat, kind="stable").astype(np.int32)
    inv_perm = np.empty_like(perm)
    inv_perm[perm] = np.arange(perm.size, dtype=np.int32)
    return counts, offsets, perm, inv_perm


# ------------------------------------------------------------------ experts
def silu(g):
    return g / (1.0 + np.exp(-g))


def _expert_weights_f64(w, e, fp8):
    """Expert e's matrix [out,in] as float64 (dequantised if fp8)."""
    if not fp8:
        return as_f64(w[e])
    q, s = codecs.quantize_rows_e4m3(as_f32(w[e]))
    return codecs.dequantize_rows_e4m3(q, s)


def expert_ffn_rows(xe, wg, wu, wd, act_rounding="none", fp8=False, taps=None):
    """One expert applied to its rows.  xe [m,H]; wg,wu [I,H]; wd [H,I], all
    float64 (weights already dequantised when fp8).  Returns y [m,H]."""
    if fp8:
        q, s = codecs.quantize_rows_e4m3(xe.astype(np.float32))
        xe = codecs.dequantize_rows_e4m3(q, s)
    g = xe @ wg.T
    u = xe @ wu.T
    a = silu(g) * u
    if fp8 or act_rounding == "bf16":
        a = codecs.f64_to_bf16_value(a)
    if taps is not None:
        taps["act"] = a
    if fp8:
        q, s = codecs.quantize_rows_e4m3(a.astype(np.float32))
        if taps is not None:
            taps["act_q"] = q
            taps["act_scale"] = s
        a = codecs.dequantize_rows_e4m3(q, s)
    return a @ wd.T


def down_project(act_rows, w_down, e, fp8=False):
    """Second expert GEMM alone: y = Wd_e a for given activations a [m,I] (float64 values)."""
    return np.asarray(act_rows, dtype=np.float64) @ _expert_weights_f64(w_down, e, fp8).T


# ------------------------------------------------------------------ the layer
def moe_layer(x, w_router, w_gate, w_up, w_down, k, bias=None, *,
              act_rounding="none", fp8=False, tokens=None, routing_logits=None,
              keep_act=False, progress=None):
    """The whole block.  Shapes: x [T,H]; w_router [E,H]; w_gate,w_up [E,I,H];
    w_down [E,H,I]; bias [E] or None.

    tokens          optional 1-D index array: the expert FFN and the combine
                    are evaluated for these tokens only (rows are independent);
                    routing and grouping are always computed for all T.
    routing_logits  optional [T,E] logits to route on instead of the float64
                    ones (used to check integer outputs against selection on a
                    device's own float32 logits).
    progress        optional callable, called with the expert index after each
                    expert has been evaluated (long runs report where they are).
    Returns a dict: logits, topk_idx, topk_w, counts, offsets, perm, inv_perm,
    out [len(tokens) or T, H], tokens; with keep_act also act/y per routed row
    of the evaluated tokens, in (token, slot) order."""
    E = np.asarray(w_router).shape[0]
    T = np.asarray(x).shape[0]
    logits = router_logits(x, w_router, bias)
    l_route = logits if routing_logits is None else np.asarray(routing_logits, dtype=np.float64)
    idx = select_topk(l_route, k)
    w = topk_weights(l_route, idx)
    counts, offsets, perm, inv_perm = group_by_expert(idx, E)

    tok = np.arange(T) if tokens is None else np.asarray(tokens, dtype=np.int64)
    H = np.asarray(x).shape[1]
    x_tok = as_f64(np.asarray(x)[tok])
    y = np.zeros((tok.size, k, H), dtype=np.float64)
    act = None
    sel = idx[tok]                                   # [n,k]
    for e in np.unique(sel):
        r, j = np.nonzero(sel == e)
        wg = _expert_weights_f64(w_gate, e, fp8)
        wu = _expert_weights_f64(w_up, e, fp8)
        wd = _expert_weights_f64(w_down, e, fp8)
        taps = {} if keep_act else None
        y[r, j] = expert_ffn_rows(x_tok[r], wg, wu, wd, act_rounding, fp8, taps)
        if keep_act:
            if act is None:
                act = np.zeros((tok.size, k, wg.shape[0]), dtype=np.float64)
            act[r, j] = taps["act"]
        if progress is not None:
            progress(int(e))
    out = np.einsum("tj,tjh->th", w[tok], y)
    res = dict(logits=logits, topk_idx=idx, topk_w=w, counts=counts, offsets=offsets,
               perm=perm, inv_perm=inv_perm, out=out, tokens=tok)
    if keep_act:
        res["act"] = act
        res["y"] = y
    return res


def ffn_flops(rows, H, I):
    """Counted work: 6*H*I flop per routed (token, expert) row."""
    return 6.0 * H * I * rows
