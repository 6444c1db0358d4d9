"""Brute-force twins of the oracle (test infrastructure only).

moe_layer_loops   pure-Python scalar loops, for inputs of a few dozen numbers
moe_layer_c       the same block as plain C triple loops in double precision
                  (brute_moe.c, built by build_c()), fast enough for the tiny
                  layer (T=256, H=256, E=8, k=2, I=512)

Both follow the block as Sec. 2.3 of the paper states it: route each token to
its top-k experts, run each expert's two-layer MLP, sum the weighted outputs.
They use no numpy routine on the data path (no matmul, no sort), so they pin
the vectorised oracle against an independent evaluation order.
"""
import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libbrute_moe.so")


def moe_layer_loops(x, w_router, w_gate, w_up, w_down, k, bias=None):
    x = [[float(v) for v in row] for row in x]
    T, H = len(x), len(x[0])
    E = len(w_router)
    I = len(w_gate[0])
    out = [[0.0] * H for _ in range(T)]
    all_idx, all_w = [], []
    for t in range(T):
        l = []
        for e in range(E):
            s = 0.0
            for h in range(H):
                s += x[t][h] * float(w_router[e][h])
            if bias is not None:
                s += float(bias[e])
            l.append(s)
        # selection: repeatedly take the largest remaining value, first index wins
        chosen = []
        for _ in range(k):
            best = -1
            for e in range(E):
                if e in chosen:
                    continue
                if best < 0 or l[e] > l[best]:
                    best = e
            chosen.append(best)
        m = max(l)
        p = [math.exp(v - m) for v in l]
        z = sum(p)
        p = [v / z for v in p]
        zs = sum(p[e] for e in chosen)
        w = [p[e] / zs for e in chosen]
        all_idx.append(chosen)
        all_w.append(w)
        for j, e in enumerate(chosen):
            a = []
            for i in range(I):
                g = 0.0
                u = 0.0
                for h in range(H):
                    g += float(w_gate[e][i][h]) * x[t][h]
                    u += float(w_up[e][i][h]) * x[t][h]
                a.append(g / (1.0 + math.exp(-g)) * u)
            for h in range(H):
                y = 0.0
                for i in range(I):
                    y += float(w_down[e][h][i]) * a[i]
                out[t][h] += w[j] * y
    # grouping by counting, in flat-id order
    counts = [0] * E
    for t in range(T):
        for j in range(k):
            counts[all_idx[t][j]] += 1
    offsets = [0] * (E + 1)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    cursor = offsets[:E]
    perm = [0] * (T * k)
    inv_perm = [0] * (T * k)
    for f in range(T * k):
        e = all_idx[f // k][f % k]
        perm[cursor[e]] = f
        inv_perm[f] = cursor[e]
        cursor[e] += 1
    return dict(topk_idx=np.array(all_idx, dtype=np.int32), topk_w=np.array(all_w),
                counts=np.array(counts, dtype=np.int32), offsets=np.array(offsets, dtype=np.int32),
                perm=np.array(perm, dtype=np.int32), inv_perm=np.array(inv_perm, dtype=np.int32),
                out=np.array(out))


def build_c(force=False):
    src = os.path.join(_HERE, "brute_moe.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-o", _SO, src, "-lm"])
    return _SO


def moe_layer_c(x, w_router, w_gate, w_up, w_down, k, bias=None):
    lib = ctypes.CDLL(build_c())
    dp = ctypes.POINTER(ctypes.c_double)
    ip = ctypes.POINTER(ctypes.c_int32)
    lib.brute_moe_layer.argtypes = [ctypes.c_int] * 5 + [dp] * 6 + [ip, dp, ip, ip, ip, dp]
    lib.brute_moe_layer.restype = None
    c = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    x, w_router, w_gate, w_up, w_down = map(c, (x, w_router, w_gate, w_up, w_down))
    T, H = x.shape
    E, I = w_gate.shape[0], w_gate.shape[1]
    b = c(bias) if bias is not None else np.zeros(E)
    idx = np.zeros((T, k), dtype=np.int32)
    w = np.zeros((T, k))
    counts = np.zeros(E, dtype=np.int32)
    perm = np.zeros(T * k, dtype=np.int32)
    inv_perm = np.zeros(T * k, dtype=np.int32)
    out = np.zeros((T, H))
    P = lambda a, t: a.ctypes.data_as(t)
    lib.brute_moe_layer(T, H, E, k, I, P(x, dp), P(w_router, dp), P(b, dp), P(w_gate, dp),
                        P(w_up, dp), P(w_down, dp), P(idx, ip), P(w, dp), P(counts, ip),
                        P(perm, ip), P(inv_perm, ip), P(out, dp))
    offsets = np.zeros(E + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    return dict(topk_idx=idx, topk_w=w, counts=counts, offsets=offsets, perm=perm,
                inv_perm=inv_perm, out=out)
