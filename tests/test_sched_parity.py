"""The library's scheduling round (include/moe_sched.h, a host-only routine) against the oracle
(oracle/scheduler.py) on seeded prefix-sharing request streams: assignments and matched tokens
bit-exact; loads and cost increments exact too, since the cost constants are integers and every
sum stays below 2^53."""
import json
import os

import numpy as np
import pytest

import paper_2605_02960_amd as moe
from paper_2605_02960_amd import build as moe_build
import workloads
from oracle import scheduler as sch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module", autouse=True)
def _built():
    moe_build.ensure_built()


def _pack(reqs, B):
    hashes = [moe.moe_sched_hash_blocks(p, B) for p, _ in reqs]
    offs = np.zeros(len(reqs) + 1, dtype=np.int64)
    offs[1:] = np.cumsum([len(h) for h in hashes])
    flat = np.concatenate(hashes) if hashes and offs[-1] else np.zeros(0, dtype=np.uint64)
    return flat, offs, np.array([len(p) for p, _ in reqs], dtype=np.int64), np.array([s for _, s in reqs], dtype=np.int64)


def _lib_round(h, reqs, B, T, f, a, loads):
    flat, offs, P, S = _pack(reqs, B)
    return moe.moe_sched_round(h, f, a, T, flat, offs, P, S, loads)


def _same(r_lib, loads, r_or):
    assigned, matched, delta, n_done = r_lib
    assert assigned.tolist() == r_or["assigned"]
    assert matched.tolist() == r_or["matched"]
    assert delta.tolist() == [float(d) for d in r_or["delta"]]
    assert loads.tolist() == [float(l) for l in r_or["loads"]]
    assert n_done == sum(g >= 0 for g in r_or["assigned"])


def test_hash_blocks_identify_prefixes():
    B = 16
    rng = np.random.default_rng(0)
    a = rng.integers(0, 32000, size=100, dtype=np.int32)
    ha = moe.moe_sched_hash_blocks(a, B)
    assert ha.shape == (6,) and len(set(ha.tolist())) == 6
    b = a.copy()
    b[40] += 1                                           # inside block 2
    hb = moe.moe_sched_hash_blocks(b, B)
    assert (ha[:2] == hb[:2]).all() and (ha[2:] != hb[2:]).all()
    assert (moe.moe_sched_hash_blocks(a[:95], B) == ha[:5]).all()       # a prefix has the prefix's hashes
    assert moe.moe_sched_hash_blocks(a[:15], B).size == 0
    assert (moe.moe_sched_hash_blocks(a, 8)[1::2] != ha).all()          # the block size is part of the hash
    # equal blocks under different histories are different entries
    c = np.concatenate([a[16:32], a[16:32]])
    hc = moe.moe_sched_hash_blocks(c, B)
    assert hc[0] != hc[1] and hc[0] != ha[1]
    # no collisions over a large set of distinct blocks
    big = moe.moe_sched_hash_blocks(rng.integers(0, 4, size=16 * 200000, dtype=np.int32), B)
    assert len(np.unique(big)) == big.size


def test_hand_worked_trace():
    g = json.load(open(os.path.join(GOLDEN, "scheduling_round_trace.json")))
    B = g["block_tokens"]
    h = moe.moe_sched_create(g["n_gpus"], B)
    try:
        for i, prefix in g["committed"]:
            moe.moe_sched_blocks_stored(h, i, moe.moe_sched_hash_blocks(prefix, B))
        reqs = [(q["prefix"], q["suffix_len"]) for q in g["requests"]]
        loads = np.zeros(g["n_gpus"])
        assigned, matched, delta, n_done = _lib_round(h, reqs, B, g["threshold"], g["f_tok"], g["f_attn"], loads)
        assert assigned.tolist() == g["expect"]["assigned"]
        assert matched.tolist() == g["expect"]["matched"]
        assert delta.tolist() == g["expect"]["delta"]
        assert loads.tolist() == g["expect"]["loads"]
        assert n_done == 7
        assert moe.moe_sched_table_size(h, 1) == (2, 5)   # [1..8] committed; pending: r0's third block, r4's block, r6's three
        assert moe.moe_sched_table_size(h, 0) == (0, 3)
    finally:
        moe.moe_sched_destroy(h)


@pytest.mark.parametrize("seed,N,B,T,f,a", [
    (0, 8, 16, 300_000_000, 44_000, 3),
    (1, 8, 16, 900_000_000, 44_000, 3),
    (2, 4, 16, 400_000_000, 44_000, 0),
    (3, 16, 32, 40_000_000, 9_000, 1),
    (4, 3, 1, 200_000, 1_000, 1),
])
def test_rounds_match_oracle_with_cache_events_between(seed, N, B, T, f, a):
    """Three rounds over one stream, with the engine's events between them: after each round
    every routed prefix is reported stored (pending -> committed), and before the last round a
    few blocks are evicted on every worker (a gap in the middle of a prefix included)."""
    reqs = workloads.generate_requests(360 if B > 1 else 60, 20, seed=seed,
                                       **({} if B > 1 else dict(root_len=(8, 40), tail_len=(4, 80), suffix_len=(1, 30))))
    reqs_or = [(p.tolist(), s) for p, s in reqs]
    tables = sch.BlockTables(N, B)
    h = moe.moe_sched_create(N, B)
    try:
        per = len(reqs) // 3
        queue = []
        for rnd in range(3):
            queue = queue + list(range(rnd * per, (rnd + 1) * per))      # left-over requests stay at the head
            loads = np.zeros(N)
            r_lib = _lib_round(h, [reqs[q] for q in queue], B, T, f, a, loads)
            r_or = sch.schedule_round(tables, [reqs_or[q] for q in queue], T, f, a)
            _same(r_lib, loads, r_or)
            for i in range(N):
                if r_or["saturated"][i]:
                    assert T <= loads[i] <= T + r_or["last_delta"][i]
            # step 2 of the round: executed prefixes become resident
            for q, g_ in zip(queue, r_or["assigned"]):
                if g_ >= 0:
                    tables.stored(g_, tables.blocks_of(reqs_or[q][0]))
                    moe.moe_sched_blocks_stored(h, g_, moe.moe_sched_hash_blocks(reqs[q][0], B))
            queue = [q for q, g_ in zip(queue, r_or["assigned"]) if g_ < 0]
            if rnd == 1:
                rng = np.random.default_rng(seed)
                for i in range(N):
                    for q in rng.choice(len(reqs), size=6, replace=False):
                        blocks = tables.blocks_of(reqs_or[q][0])
                        hs = moe.moe_sched_hash_blocks(reqs[q][0], B)
                        if len(blocks) >= 3:
                            j = int(rng.integers(1, len(blocks) - 1))
                            tables.evicted(i, [blocks[j]])
                            moe.moe_sched_blocks_evicted(h, i, hs[j:j + 1])
            for i in range(N):
                assert moe.moe_sched_table_size(h, i) == (len(tables.committed[i]), len(tables.pending[i]))
    finally:
        moe.moe_sched_destroy(h)


def test_starting_loads_and_saturated_workers_are_skipped():
    B = 4
    h = moe.moe_sched_create(3, B)
    try:
        reqs = [(np.arange(8, dtype=np.int32), 2)] * 3
        loads = np.array([100.0, 5.0, 100.0])
        assigned, matched, delta, n_done = _lib_round(h, reqs, B, 30.0, 1, 0, loads)
        tables = sch.BlockTables(3, B)
        r_or = sch.schedule_round(tables, [(list(range(8)), 2)] * 3, 30, 1, 0, loads=[100, 5, 100])
        _same((assigned, matched, delta, n_done), loads, r_or)
        assert assigned.tolist() == [1, 1, 1] and loads.tolist() == [100.0, 5.0 + 10 + 2 + 2, 100.0]
        # all saturated: nothing is consumed
        loads = np.array([30.0, 31.0, 1e9])
        assigned, _, _, n_done = _lib_round(h, reqs, B, 30.0, 1, 0, loads)
        assert assigned.tolist() == [-1, -1, -1] and n_done == 0 and loads.tolist() == [30.0, 31.0, 1e9]
        # empty queue
        assigned, _, _, n_done = _lib_round(h, [], B, 30.0, 1, 0, np.zeros(3))
        assert assigned.size == 0 and n_done == 0
    finally:
        moe.moe_sched_destroy(h)


def test_argument_errors_change_nothing():
    L = moe.lib()
    import ctypes
    hp = ctypes.c_void_p()
    assert L.moe_sched_create(0, 16, ctypes.byref(hp)) == -2
    assert L.moe_sched_create(4, 0, ctypes.byref(hp)) == -2
    assert L.moe_sched_create(4, 16, None) == -1
    h = moe.moe_sched_create(2, 4)
    try:
        toks = np.arange(8, dtype=np.int32)
        hs = moe.moe_sched_hash_blocks(toks, 4)
        loads = np.zeros(2)
        with pytest.raises(moe.MoEError):                # 8 prefix tokens need 2 hashes, 1 given
            moe.moe_sched_round(h, 1, 0, 10, hs[:1], [0, 1], [8], [1], loads)
        with pytest.raises(moe.MoEError):
            moe.moe_sched_round(h, -1, 0, 10, hs, [0, 2], [8], [1], loads)
        with pytest.raises(moe.MoEError):
            moe.moe_sched_round(h, 1, 0, 10, hs, [0, 2], [8], [-1], loads)
        with pytest.raises(moe.MoEError):
            moe.moe_sched_blocks_stored(h, 2, hs)
        assert loads.tolist() == [0.0, 0.0] and moe.moe_sched_table_size(h, 0) == (0, 0)
    finally:
        moe.moe_sched_destroy(h)


def test_progress_reports_match_oracle():
    f = 44_000
    B = 16
    reqs = workloads.generate_requests(50, 6, seed=11)
    reqs_or = [(p.tolist(), s) for p, s in reqs]
    tables = sch.BlockTables(4, B)
    h = moe.moe_sched_create(4, B)
    try:
        loads = np.zeros(4)
        assigned, matched, delta, n_done = _lib_round(h, reqs, B, 1e18, f, 0, loads)
        r_or = sch.schedule_round(tables, reqs_or, 10 ** 18, f, 0)
        _same((assigned, matched, delta, n_done), loads, r_or)
        want = r_or["loads"]
        rng = np.random.default_rng(0)
        for _ in range(40):
            i, tok = int(rng.integers(0, 4)), int(rng.integers(0, 3000))
            moe.moe_sched_tokens_executed(h, loads, i, tok, f)
            want = sch.tokens_executed(want, i, tok, f)
            assert loads.tolist() == [float(v) for v in want]
        assert min(loads) >= 0.0
        with pytest.raises(moe.MoEError):
            moe.moe_sched_tokens_executed(h, loads, 4, 1, f)
        with pytest.raises(moe.MoEError):
            moe.moe_sched_tokens_executed(h, loads, 0, -1, f)
    finally:
        moe.moe_sched_destroy(h)


def test_token_unit_accounting_is_the_same_round_in_other_units():
    """App. B.4's last fallback: without f_tok, the threshold and the work counters are kept in
    tokens (f_tok = 1, no attention term).  With a power-of-two f_tok every product is an exact
    scaling, so the FLOPs-unit round must make the very same assignments with loads that are
    exactly f_tok times the token-unit ones; both equal the oracle."""
    N, B = 4, 16
    reqs = workloads.generate_requests(200, 12, seed=21)
    reqs_or = [(p.tolist(), s) for p, s in reqs]
    t_tok, unit = moe.moe_resolve_threshold(0.0, 10e-3, 25e-3, 0.0, 8192, 1.2)      # no f_tok: tokens
    assert unit == 1 and t_tok == pytest.approx(1.2 * 2.5 * 8192)
    f = 2.0 ** 25
    t_fl, unit = moe.moe_resolve_threshold(0.0, 10e-3, 25e-3, f, 8192, 1.2)
    assert unit == 0 and t_fl == t_tok * f
    res = []
    for f_tok, T in ((1.0, t_tok), (f, t_fl)):
        h = moe.moe_sched_create(N, B)
        try:
            loads = np.zeros(N)
            res.append((_lib_round(h, reqs, B, T, f_tok, 0, loads), loads))
        finally:
            moe.moe_sched_destroy(h)
    (r_tok, l_tok), (r_fl, l_fl) = res
    assert r_tok[0].tolist() == r_fl[0].tolist() and r_tok[1].tolist() == r_fl[1].tolist()
    assert (r_tok[2] * f).tolist() == r_fl[2].tolist() and (l_tok * f).tolist() == l_fl.tolist()
    r_or = sch.schedule_round(sch.BlockTables(N, B), reqs_or, t_tok, 1, 0)
    _same(r_tok, l_tok, r_or)
    # in token units a request's increment is its number of uncached tokens
    P = np.array([len(p) for p, _ in reqs])
    S = np.array([s for _, s in reqs])
    done = r_tok[0] >= 0
    assert np.array_equal(r_tok[2][done], (P - r_tok[1] + S)[done].astype(np.float64))
