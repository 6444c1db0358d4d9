"""Seeded synthetic inputs for the MoE prefill block.

This module only draws random numbers and stores them in the tensors' storage
types; it holds none of the block's arithmetic and is the one module that both
the CPU oracle's tests and the HIP path's tests/bench read.  The shapes follow
the model the paper evaluates (Sec. 8.1: 128 experts, top-8 routing) and its
64K-token batches (Sec. 4.2, Fig. 4); the skewed-routing recipe stands in for
the expert imbalance reported there.  Real model weights and the paper's
datasets are not used: the block's cost depends on shapes and on the routing
histogram only.

Storage: "bf16" tensors are returned as numpy uint16 bit patterns (rounded from
the float32 draw by torch's CPU cast), float32 tensors as float32.
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
import os

import numpy as np
import torch

BASE_SEED = 260502960


@dataclass(frozen=True)
class MoEWorkload:
    name: str
    cfg_id: int
    T: int
    H: int
    E: int
    K: int
    I: int
    dtype: str            # "fp32" | "bf16" | "fp8" (fp8: bf16 master tensors, quantised by the method)
    zipf_bias: bool = False

    @property
    def rows(self):
        return self.T * self.K


TINY = MoEWorkload("tiny_fp32", 1, 256, 256, 8, 2, 512, "fp32")
QWEN3_8K = MoEWorkload("qwen3_235b_T8192_bf16", 2, 8192, 4096, 128, 8, 1536, "bf16")
QWEN3_64K_ZIPF = MoEWorkload("qwen3_235b_T65536_bf16_zipf", 3, 65536, 4096, 128, 8, 1536, "bf16", True)
QWEN3_32K_FP8 = MoEWorkload("qwen3_235b_T32768_fp8", 4, 32768, 4096, 128, 8, 1536, "fp8")
# Second shape: the 30B-A3B sibling of the same model family (the model behind the paper's
# motivation figures, Sec. 3); its dimensions come from the public model configuration:
# hidden 2048, expert intermediate 768, 128 experts, top-8.
QWEN3_30B_64K_ZIPF = MoEWorkload("qwen3_30b_a3b_T65536_bf16_zipf", 6, 65536, 2048, 128, 8, 768, "bf16", True)
SWEEP_T = (512, 1024, 2048, 4096, 8192, 16384, 32768, 65536, 131072)

CONFIGS = {w.name: w for w in (TINY, QWEN3_8K, QWEN3_64K_ZIPF, QWEN3_32K_FP8, QWEN3_30B_64K_ZIPF)}


def sweep_point(T):
    return replace(QWEN3_8K, name=f"qwen3_235b_T{T}_bf16_sweep", cfg_id=5, T=T)


def scaled(w, **kw):
    """Same recipe at other sizes (for parity cases the oracle finishes quickly)."""
    return replace(w, **kw)


def _to_storage(a32, dtype):
    if dtype == "fp32":
        return a32
    t = torch.from_numpy(a32).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _normal(seed_words, shape, sigma, dtype):
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence(seed_words)))
    a = rng.standard_normal(shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return _to_storage(a, dtype)


def zipf_bias(E):
    """b_e = 1.5 * ln(1/(e+1)), e = 0-based expert index, float32."""
    e = np.arange(E, dtype=np.float64)
    return (1.5 * np.log(1.0 / (e + 1.0))).astype(np.float32)


def generate_x(w, seed=0, threads=None):
    """Only the activations x [T,H] of `generate` (same values)."""
    st = "fp32" if w.dtype == "fp32" else "bf16"
    base = [BASE_SEED, w.cfg_id, seed]
    threads = threads or min(16, os.cpu_count() or 1)
    x = np.empty((w.T, w.H), dtype=np.float32 if st == "fp32" else np.uint16)
    chunk = 2048

    def fill_x(c):
        n = min(chunk, w.T - c)
        x[c:c + n] = _normal(base + [0, c], (n, w.H), 1.0, st)

    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(fill_x, range(0, w.T, chunk)))
    return x


def generate(w, seed=0, threads=None):
    """All tensors of one layer.  Keys: x [T,H]; w_router [E,H] float32; bias [E]
    float32 or None; w_gate, w_up [E,I,H]; w_down [E,H,I].  x and the expert
    weights are in the workload's storage type (fp8 workloads: bf16 masters)."""
    st = "fp32" if w.dtype == "fp32" else "bf16"
    base = [BASE_SEED, w.cfg_id, seed]
    threads = threads or min(16, os.cpu_count() or 1)
    out = {}
    sto = np.float32 if st == "fp32" else np.uint16
    out["w_router"] = _normal(base + [1], (w.E, w.H), 0.02, "fp32")
    out["bias"] = zipf_bias(w.E) if w.zipf_bias else None
    x = generate_x(w, seed, threads)
    wg = np.empty((w.E, w.I, w.H), dtype=sto)
    wu = np.empty((w.E, w.I, w.H), dtype=sto)
    wd = np.empty((w.E, w.H, w.I), dtype=sto)
    def fill_e(e):
        wg[e] = _normal(base + [2, e], (w.I, w.H), 0.02, st)
        wu[e] = _normal(base + [3, e], (w.I, w.H), 0.02, st)
        wd[e] = _normal(base + [4, e], (w.H, w.I), 0.02, st)

    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(fill_e, range(w.E)))
    out.update(x=x, w_gate=wg, w_up=wu, w_down=wd)
    return out


def generate_requests(n_requests, n_prefixes, seed=0, *, n_roots=4, root_len=(256, 1024),
                      tail_len=(64, 2048), suffix_len=(16, 512), zipf_s=1.1, vocab=32000):
    """A prefix-sharing request stream for the frontend's scheduling round (Sec. 7; the
    stand-in for the prefix-sharing evaluation sets of Sec. 8.1, which are not used).

    n_prefixes distinct prompts' prefixes, each one of n_roots shared roots followed by its own
    tail (so two prefixes under one root share the root's blocks only); every request draws its
    prefix with Zipf(zipf_s) popularity and a suffix length uniformly from suffix_len.  Lengths
    are not multiples of the block size on purpose.  Returns a list of
    (prefix_tokens int32 array, suffix_len int) in arrival order."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED, 7, seed])))
    roots = [rng.integers(0, vocab, size=int(rng.integers(root_len[0], root_len[1] + 1)), dtype=np.int32)
             for _ in range(n_roots)]
    prefixes = []
    for j in range(n_prefixes):
        tail = rng.integers(0, vocab, size=int(rng.integers(tail_len[0], tail_len[1] + 1)), dtype=np.int32)
        prefixes.append(np.concatenate([roots[j % n_roots], tail]))
    p = 1.0 / np.arange(1, n_prefixes + 1, dtype=np.float64) ** zipf_s
    pick = rng.choice(n_prefixes, size=n_requests, p=p / p.sum())
    sfx = rng.integers(suffix_len[0], suffix_len[1] + 1, size=n_requests)
    return [(prefixes[int(j)], int(s)) for j, s in zip(pick, sfx)]
