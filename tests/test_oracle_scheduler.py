"""Pins of the scheduling-round oracle (oracle/scheduler.py) against what the paper and plain
arithmetic fix: the closed-form examples of Sec. 7.3, the load interval of Sec. 7.4, the
tie-breaking and stopping rules of Alg. 1 (App. A), block-granular matching (Sec. 7.2) and a
hand-worked trace stored under tests/golden/."""
import json
import os

import numpy as np
import pytest

import workloads
from oracle import scheduler as sch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _toks(*parts):
    return [t for p in parts for t in p]


def test_cost_terms_closed_forms():
    # Eq. 2 with the whole prefix cached: only the suffix cost is left (Sec. 7.3)
    f, a = 1000, 3
    P, S = 4096, 100
    assert sch.cost_delta(P, P, S, f, a) == sch.c_sfx(S, P, f, a)
    # no attention term: Delta = uncached tokens * f_tok (App. B.2)
    assert sch.cost_delta(P, 1024, S, f, 0) == (P - 1024 + S) * f
    # attention pairs: a request with nothing cached costs exactly causal attention over P+S tokens
    n = P + S
    assert sch.cost_delta(P, 0, S, 0, 1) == n * (n + 1) // 2
    # and partial caching removes the pairs among the cached tokens' queries only through C_pfx's argument
    assert sch.cost_delta(P, 0, S, f, a) - sch.cost_delta(P, P, S, f, a) == sch.c_pfx(P, f, a)


def test_ten_same_prefix_requests_cost_one_prefix_pass():
    """Sec. 7.3: ten requests sharing a 4096-token prefix cost one prefix pass plus ten suffix
    passes on the GPU that takes them all, not ten full requests."""
    B, P, S, f = 16, 4096, 64, 7
    prefix = list(range(P))
    t = sch.BlockTables(4, B)
    r = sch.schedule_round(t, [(prefix, S)] * 10, threshold=10 ** 12, f_tok=f, f_attn=0)
    assert r["assigned"] == [0] * 10                     # the first goes to GPU 0 (all empty), the rest follow the match
    assert r["matched"] == [0] + [P] * 9
    assert r["loads"][0] == f * (P + 10 * S)
    assert r["loads"][0] < f * 10 * (P + S)
    assert r["loads"][1:] == [0, 0, 0]


def test_no_sharing_is_round_robin_until_saturation():
    """Distinct prompts of equal cost c: no GPU ever matches, so the tie rule sends each request
    to the least-loaded GPU (lowest index among equals): round robin, ceil(T/c) requests per
    GPU, and the round stops with the rest of the queue untouched."""
    N, B, c_tok, f = 3, 16, 160, 5
    c = c_tok * f
    T = 4 * c - 1                                        # saturates with the 4th request
    reqs = [([1000 * j + k for k in range(c_tok - 10)], 10) for j in range(20)]
    r = sch.schedule_round(sch.BlockTables(N, B), reqs, T, f, 0)
    assert r["assigned"][:12] == [0, 1, 2] * 4
    assert r["assigned"][12:] == [-1] * 8
    assert r["loads"] == [4 * c] * 3 and all(r["saturated"])


def test_load_interval_after_saturation():
    """Sec. 7.4: GPUs are retired one at a time, so a saturated GPU ends in [T, T + Delta_last];
    an unsaturated one (queue ran dry) is below T."""
    seen_sat = seen_unsat = seen_left = False
    for seed in range(3):
        reqs = [(p.tolist(), s) for p, s in workloads.generate_requests(200, 24, seed=seed)]
        f, a = 44_000, 3
        for T in (300_000_000, 900_000_000):
            r = sch.schedule_round(sch.BlockTables(8, 16), reqs, T, f, a)
            for i in range(8):
                if r["saturated"][i]:
                    assert T <= r["loads"][i] <= T + r["last_delta"][i]
                else:
                    assert r["loads"][i] < T
            n_assigned = sum(g >= 0 for g in r["assigned"])
            assert all(r["saturated"]) or n_assigned == len(reqs)
            # the assigned requests are a prefix of the queue (FIFO drain), and loads add up
            assert all(g >= 0 for g in r["assigned"][:n_assigned]) and all(g < 0 for g in r["assigned"][n_assigned:])
            for i in range(8):
                assert r["loads"][i] == sum(d for g, d in zip(r["assigned"], r["delta"]) if g == i)
            seen_sat |= any(r["saturated"])
            seen_unsat |= not all(r["saturated"])
            seen_left |= n_assigned < len(reqs)
    assert seen_sat and seen_unsat and seen_left         # the cases above exercise both ends


def test_block_granularity_and_contiguity():
    B = 16
    t = sch.BlockTables(1, B)
    base = list(range(100, 100 + 80))                    # 5 full blocks
    t.promise(0, base)
    assert t.block_match(0, base) == 80
    assert t.block_match(0, base[:79]) == 64             # a partial last block never counts
    other = list(base)
    other[40] = -1                                       # differs inside block 2
    assert t.block_match(0, other) == 32
    other = list(base)
    other[0] = -1                                        # first block differs: later equal blocks do not count
    assert t.block_match(0, other) == 0
    # eviction of a middle block cuts the contiguous run
    t.stored(0, t.blocks_of(base))
    t.evicted(0, [t.blocks_of(base)[2]])
    assert t.block_match(0, base) == 32


def test_longest_match_beats_load_and_ties_go_to_lighter_gpu():
    B, f = 4, 1
    shared = list(range(8))
    t = sch.BlockTables(3, B)
    t.stored(0, t.blocks_of(shared))                     # GPU 0 holds 2 blocks
    t.stored(1, t.blocks_of(shared[:4]))                 # GPU 1 holds 1 block
    req = (shared + [50, 51, 52, 53], 2)
    # GPU 0 is the most loaded but has the longest match
    r = sch.schedule_round(t, [req], 1000, f, 0, loads=[500, 10, 0])
    assert r["assigned"] == [0] and r["matched"] == [8] and r["delta"] == [4 + 2]
    # equal matches (GPU 0 and GPU 1 both hold everything now): the lighter one wins
    t.stored(1, t.blocks_of(req[0]))
    t.stored(0, t.blocks_of(req[0]))
    r = sch.schedule_round(t, [req], 1000, f, 0, loads=[500, 10, 0])
    assert r["assigned"] == [1] and r["matched"] == [12]
    # no positive match anywhere: least-loaded GPU (App. B.2 fallback)
    r = sch.schedule_round(t, [([9] * 8, 1)], 1000, f, 0, loads=[500, 10, 0])
    assert r["assigned"] == [2]


def test_popular_prefix_spills_to_next_best_match():
    """Sec. 7.4: once the primary GPU is saturated the same rule sends the prefix to the GPU
    with the next-best match; saturated GPUs are never evaluated."""
    B, f = 4, 1
    root, tail = list(range(8)), list(range(100, 108))
    t = sch.BlockTables(3, B)
    t.stored(2, t.blocks_of(root))                       # GPU 2 already holds the root only
    reqs = [(root + tail, 4)] * 6
    T = 30
    r = sch.schedule_round(t, reqs, T, f, 0)
    # 1st: GPU 2 (match 8): 8+4=12; 2nd..: GPU 2 (match 16): +4 each -> 16, 20, 24, 28, 32>=30 saturates at the 6th
    assert r["assigned"] == [2] * 6 and r["loads"][2] == 32
    r = sch.schedule_round(t, reqs, T, f, 0, loads=[0, 5, 28])
    # 1st saturates GPU 2 (28+4); afterwards nobody else matches: the lighter of GPUs 0/1 takes the whole
    # prompt (20), keeps the prefix (pending entries count for the match) until it saturates too (32),
    # and the last request spills once more, to GPU 1
    assert r["assigned"] == [2, 0, 0, 0, 0, 1]
    assert r["matched"] == [16, 0, 16, 16, 16, 0]
    assert r["loads"] == [32, 25, 32]


def test_saturated_at_start_and_empty_queue():
    t = sch.BlockTables(2, 16)
    r = sch.schedule_round(t, [([1] * 32, 1)], 10, 1, 0, loads=[10, 11])
    assert r["assigned"] == [-1] and r["loads"] == [10, 11]
    r = sch.schedule_round(t, [], 10, 1, 0)
    assert r["assigned"] == [] and r["loads"] == [0, 0]


def test_hand_worked_trace():
    """A trace worked by hand from Alg. 1 (stored with its derivation in the fixture)."""
    g = json.load(open(os.path.join(GOLDEN, "scheduling_round_trace.json")))
    t = sch.BlockTables(g["n_gpus"], g["block_tokens"])
    for i, prefix in g["committed"]:
        t.stored(i, t.blocks_of(prefix))
    reqs = [(q["prefix"], q["suffix_len"]) for q in g["requests"]]
    r = sch.schedule_round(t, reqs, g["threshold"], g["f_tok"], g["f_attn"])
    assert r["assigned"] == g["expect"]["assigned"]
    assert r["matched"] == g["expect"]["matched"]
    assert r["delta"] == g["expect"]["delta"]
    assert r["loads"] == g["expect"]["loads"]


def test_counter_is_drift_free_with_one_constant():
    """App. B.3: with f_attn = 0 a request adds u * f_tok at routing time and the engine's progress
    reports take tokens * f_tok away again; once every uncached token has been executed the
    counter is back at zero exactly, and it never goes below zero."""
    f = 44_000
    t = sch.BlockTables(2, 16)
    prefix = list(range(100))
    r = sch.schedule_round(t, [(prefix, 20), (prefix, 7), ([5] * 40, 3)], 10 ** 12, f, 0)
    assert r["assigned"] == [0, 0, 1]
    uncached = [100 + 20, (100 - 96) + 7, 40 + 3]            # the sibling re-uses 6 full blocks = 96 tokens
    assert r["delta"] == [u * f for u in uncached]
    loads = r["loads"]
    loads = sch.tokens_executed(loads, 0, 64, f)
    loads = sch.tokens_executed(loads, 0, uncached[0] + uncached[1] - 64, f)
    loads = sch.tokens_executed(loads, 1, uncached[2], f)
    assert loads == [0, 0]
    assert sch.tokens_executed(loads, 1, 5, f) == [0, 0]
