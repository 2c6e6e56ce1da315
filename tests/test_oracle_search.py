"""Pins for the oracle of the offline pattern search (Kernel-Aware Sparse Pattern Search, Alg. 1)."""
import numpy as np
import pytest

from harness import gen
from oracle import oracle as orc
from oracle import search as srch
from helpers import numpy_mask

T, IS, BC = 0, 1, 2


def _scores(Q, K, b, w):
    return [x.astype(np.float32) for x in orc.estimate(Q, K, b, w)]


def _pairs_by_numpy(v, s, blk, N, b, w, sink, p, x):
    """|M| of candidate (p, x) of head 0, counted on the boolean mask (independent of masked_rows)."""
    bud = srch.candidate_budgets(p, x, N, b, sink)
    ix = orc.build_index(v[:1], s[:1], blk[:1], N, b, w, bud, override=[p])
    return int(numpy_mask(N, b, ix, 0).sum())


def test_refine_finds_the_size_closest_to_the_target():
    # brute force over the whole search space of every candidate on a tiny head
    Hq, Hkv, N, b, w, sink = 1, 1, 256, 64, 32, 1
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=71)
    v, s, blk = _scores(Q, K, b, w)
    for p in (T, IS, BC):
        lo, hi = srch.candidate_range(p, N, b)
        table = {x: _pairs_by_numpy(v, s, blk, N, b, w, sink, p, x) for x in range(lo, hi + 1)}
        vals = [table[x] for x in range(lo, hi + 1)]
        assert all(a <= c for a, c in zip(vals, vals[1:])), (p, vals)   # monotone in the size
        assert vals[-1] == N * (N + 1) // 2 or p == T and vals[-1] == N * (N + 1) // 2
        for target in (0, vals[0], (vals[0] + vals[-1]) // 2, vals[len(vals) // 2] + 1, vals[-1], 10 ** 9):
            x, pairs = srch.refine(lambda x: table[x], lo, hi, target, 0)
            assert pairs == table[x]
            assert abs(pairs - target) == min(abs(t - target) for t in vals), (p, target, x)
        # with a tolerance the first probe inside it is accepted
        mid = (lo + hi) // 2
        x, pairs = srch.refine(lambda x: table[x], lo, hi, table[mid], 0)
        assert pairs == table[mid]


def test_triangular_pairs_closed_form():
    Hq, Hkv, N, b, w, sink = 1, 1, 512, 64, 32, 2
    nb = N // b
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=72)
    v, s, blk = _scores(Q, K, b, w)
    for x in (1, 2, 3, 5, nb):
        want = 0
        for i in range(N):
            R = i // b
            band = min(x - 1, R)                         # blocks R-x+1 .. R-1
            sinks = max(0, min(sink, R - x + 1))         # sink blocks left of the band
            want += (i % b) + 1 + b * (band + sinks)
        bud = srch.candidate_budgets(T, x, N, b, sink)
        ix = orc.build_index(v, s, blk, N, b, w, bud, override=[T])
        assert int(orc.masked_rows(Q, K, V, b, ix)[2].sum()) == want


def test_full_target_makes_every_candidate_dense():
    Hq, Hkv, N, b, w = 2, 1, 256, 64, 32
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=73)
    v, s, blk = _scores(Q, K, b, w)
    full = N * (N + 1) // 2
    res = srch.search_patterns(Q, K, V, v, s, blk, b, w, 1, full, 0)
    for r in res:
        assert r["pairs"] == [full] * 3
        assert max(r["err"]) <= 1e-9
        lo_hi = [srch.candidate_range(p, N, b) for p in (T, IS, BC)]
        assert r["param"][0] == lo_hi[0][1] and r["param"][2] == lo_hi[2][1]


def test_planted_heads_are_given_a_pattern_that_expresses_them():
    # one head per planted structure, budget 0.4 of the causal pairs.  The candidate that can
    # express the structure loses the least of the dense output: scattered columns and diagonals
    # need Interval-Slash, hot blocks need Block-Cluster; a sink + band head is served by the static
    # band and by the block selection (which finds the same blocks by itself), not by a few
    # diagonals.  An argmax in place of the argmin, or errors attached to the wrong candidate,
    # fail here.
    wl = gen.scaled(gen.WORKLOADS["cfg2"], seq_len=1024, n_q_heads=3, n_kv_heads=1, block=64,
                    last_q=64, n_cols=24, n_offs=12, n_hot=24, hot_block=64, window=192, n_sinks=4,
                    seed=74)
    data = gen.generate(wl)
    Q, K, V = data["Q"], data["K"], data["V"]
    N, b, w = wl.seq_len, wl.block, wl.last_q
    v, s, blk = _scores(Q, K, b, w)
    target = N * (N + 1) // 2 * 2 // 5
    res = srch.search_patterns(Q, K, V, v, s, blk, b, w, 1, target, target // 50)
    planted = [pl.pattern for pl in data["plants"]]
    assert planted == [T, IS, BC]
    assert res[0]["pattern"] in (T, BC) and res[0]["err"][T] < res[0]["err"][IS]
    assert res[1]["pattern"] == IS and res[2]["pattern"] == BC
    for r in res:
        assert r["pattern"] == int(np.argmin(r["err"])) and all(e > 0 for e in r["err"])
        # every refined candidate sits at the target within what its granularity allows
        assert all(abs(pr - target) <= max(target // 50, N * b) for pr in r["pairs"])
