"""Pins for index selection (Alg. 2 TopK / CombineIndices, Alg. 3 TopKBlocks,
the per-head pattern rule and the default budgets)."""
import itertools
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from harness import gen
from oracle import oracle as orc

T, IS, BC = 0, 1, 2


def _bud(**kw):
    d = dict(sink_blocks=1, local_blocks=1, k_vertical=3, k_slash=2, k_blocks=13)
    d.update(kw)
    return orc.Budgets(**d)


def _brute_topk(score, k):
    """Lexicographically smallest index set among those of maximal total score."""
    best, best_sum = None, None
    sc = [float(x) for x in score]          # fp32 values: sums of a few are exact in fp64
    for comb in itertools.combinations(range(len(sc)), k):
        t = sum(sc[c] for c in comb)
        if best is None or t > best_sum:
            best, best_sum = comb, t
    return np.array(best, np.int32)


def test_topk_brute_force_seq64():
    # seq_len 64 end to end: scores from the estimator, all three selections by enumeration
    N, b, w = 64, 8, 8
    Q, K, _ = gen.random_qkv(2, 1, N, 128, seed=64)
    v, s, blk = (x.astype(np.float32) for x in orc.estimate(Q, K, b, w))
    nb = N // b
    bud = _bud(k_vertical=3, k_slash=2, k_blocks=nb + 4)
    for h in range(2):
        ix = orc.build_index(v, s, blk, N, b, w, bud, override=[IS, IS])
        assert (ix.cols[h] == _brute_topk(v[h], 3)).all()
        assert (ix.offs[h] == _brute_topk(s[h], 2)).all()
        ix = orc.build_index(v, s, blk, N, b, w, bud, override=[BC, BC])
        cand = [(R, C) for R in range(nb) for C in range(R)]
        sel = _brute_topk([blk[h, R, C] for R, C in cand], 4)
        want = {cand[t] for t in sel} | {(R, R) for R in range(nb)}
        got = {(R, int(C)) for R in range(nb)
               for C in ix.blkcols[h, ix.rowptr[h, R]:ix.rowptr[h, R + 1]]}
        assert got == want


def _stable_topk(score, k):
    bits = np.asarray(score, np.float32).view(np.uint32).astype(np.int64)
    return np.sort(np.argsort(-bits, kind="stable")[:k]).astype(np.int32)


@settings(max_examples=60, deadline=None)
@given(st.lists(st.integers(0, 4), min_size=16, max_size=16), st.integers(1, 7),
       st.lists(st.integers(0, 3), min_size=16, max_size=16), st.integers(1, 5))
def test_topk_ties_go_to_lower_index(vs, kv, ss, ks):
    N, b, w = 16, 4, 4
    v = np.array([vs], np.float32)
    s = np.array([ss], np.float32)
    blk = np.zeros((1, 4, 4), np.float32)
    ix = orc.build_index(v, s, blk, N, b, w, _bud(k_vertical=kv, k_slash=ks, k_blocks=4),
                         override=[IS])
    assert (ix.cols[0] == _stable_topk(v[0], kv)).all()
    assert (ix.offs[0] == _stable_topk(s[0], ks)).all()
    if kv <= 4:
        assert (ix.cols[0] == _brute_topk(v[0], kv)).all()


@settings(max_examples=40, deadline=None)
@given(st.lists(st.integers(0, 3), min_size=36, max_size=36), st.integers(6, 21))
def test_block_topk_ties_and_csr_invariants(vals, kb):
    nb, b = 6, 4
    N = nb * b
    blk = np.array(vals, np.float32).reshape(1, nb, nb)
    v = np.ones((1, N), np.float32)
    ix = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=kb), override=[BC])
    cand = [(R, C) for R in range(nb) for C in range(R)]
    flat = np.array([R * nb + C for R, C in cand])
    sel = _stable_topk([blk[0, R, C] for R, C in cand], kb - nb)
    want = sorted(list(flat[sel]) + [R * nb + R for R in range(nb)])
    rp = ix.rowptr[0]
    got = [R * nb + int(C) for R in range(nb) for C in ix.blkcols[0, rp[R]:rp[R + 1]]]
    assert got == want
    assert rp[0] == 0 and (np.diff(rp) >= 1).all() and rp[nb] == len(want) == kb
    for R in range(nb):
        row = ix.blkcols[0, rp[R]:rp[R + 1]]
        assert (np.diff(row) > 0).all() and row[-1] == R
    assert (ix.blkcols[0, rp[nb]:] == -1).all()


def _row_share(kb, nb, R):
    """Blocks kept in row R by the per-row rule, written with exact fractions."""
    from fractions import Fraction
    import math
    return min(R + 1, math.ceil(Fraction(kb * (R + 1), nb * (nb + 1) // 2)))


@settings(max_examples=40, deadline=None)
@given(st.lists(st.integers(0, 3), min_size=36, max_size=36), st.integers(6, 21))
def test_per_row_block_topk_ties_and_csr_invariants(vals, kb):
    # per-row reading of TopKBlocks: every row keeps its share by a stable per-row sort
    nb, b = 6, 4
    N = nb * b
    blk = np.array(vals, np.float32).reshape(1, nb, nb)
    v = np.ones((1, N), np.float32)
    ix = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=kb, block_select=1), override=[BC])
    rp = ix.rowptr[0]
    total = 0
    for R in range(nb):
        keep = _row_share(kb, nb, R)
        want = sorted(list(_stable_topk(blk[0, R, :R], keep - 1)) + [R])
        assert list(ix.blkcols[0, rp[R]:rp[R + 1]]) == want
        total += keep
    assert rp[0] == 0 and rp[nb] == total <= kb + nb
    assert total >= kb                      # shares are rounded up
    assert (ix.blkcols[0, rp[nb]:] == -1).all()


def test_per_row_block_topk_brute_force_and_limits():
    rng = np.random.default_rng(5)
    nb, b = 8, 4
    N = nb * b
    blk = rng.random((1, nb, nb)).astype(np.float32)
    v = np.ones((1, N), np.float32)
    kb = 18                                  # half of the 36 causal blocks
    ix = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=kb, block_select=1), override=[BC])
    rp = ix.rowptr[0]
    for R in range(nb):
        keep = _row_share(kb, nb, R)
        assert keep == -(-(R + 1) // 2)      # ceil(half of the row's R+1 causal blocks)
        row = ix.blkcols[0, rp[R]:rp[R + 1]]
        assert len(row) == keep and row[-1] == R
        if keep > 1:
            assert (row[:-1] == _brute_topk(blk[0, R, :R], keep - 1)).all()
    # k_blocks = nb: 8/36 of every row rounded up; k_blocks = all causal blocks: everything
    ix = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=nb, block_select=1), override=[BC])
    assert list(np.diff(ix.rowptr[0])) == [1, 1, 1, 1, 2, 2, 2, 2]
    ix = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=36, block_select=1), override=[BC])
    assert (np.diff(ix.rowptr[0]) == np.arange(1, nb + 1)).all()
    # the other patterns do not depend on the block rule
    a = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=kb, block_select=0), override=[T])
    c = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=kb, block_select=1), override=[T])
    assert (a.rowptr == c.rowptr).all() and (a.blkcols[0, :a.rowptr[0, -1]] == c.blkcols[0, :c.rowptr[0, -1]]).all()


def _csr_pairs(ix, h, nb):
    rp = ix.rowptr[h]
    return {(R, int(C)) for R in range(nb) for C in ix.blkcols[h, rp[R]:rp[R + 1]]}


@pytest.mark.parametrize("seed,N,b,ks", [(0, 96, 8, 3), (1, 128, 16, 5), (2, 64, 4, 64)])
def test_block_widened_diagonals_are_the_smallest_block_cover(seed, N, b, ks):
    # the kept block pairs are exactly those that hold a (query, key) pair of a selected diagonal,
    # plus the diagonal blocks: every exact pair is covered, no block is kept without one
    rng = np.random.default_rng(seed)
    nb = N // b
    v = rng.random((2, N)).astype(np.float32)
    s = rng.random((2, N)).astype(np.float32)
    blk = np.zeros((2, nb, nb), np.float32)
    exact = orc.build_index(v, s, blk, N, b, 4, _bud(k_slash=ks, k_blocks=nb), override=[IS, IS])
    wide = orc.build_index(v, s, blk, N, b, 4, _bud(k_slash=ks, k_blocks=nb, diagonal_select=1),
                           override=[IS, IS])
    assert (wide.n_offs == 0).all() and (wide.offs == -1).all()
    assert (wide.cols == exact.cols).all() and (wide.pattern == exact.pattern).all()
    i = np.arange(N)
    for h in range(2):
        offs = exact.offs[h, :exact.n_offs[h]]
        want = {(R, R) for R in range(nb)}
        ii, oo = np.meshgrid(i, offs, indexing="ij")
        ok = ii >= oo
        want |= set(zip((ii[ok] // b).tolist(), ((ii[ok] - oo[ok]) // b).tolist()))
        got = _csr_pairs(wide, h, nb)
        assert got == want
        rp = wide.rowptr[h]
        for R in range(nb):
            row = wide.blkcols[h, rp[R]:rp[R + 1]]
            assert (np.diff(row) > 0).all() and row[-1] == R
        assert (wide.blkcols[h, rp[nb]:] == -1).all()


def test_block_widened_diagonals_special_cases():
    rng = np.random.default_rng(9)
    N, w = 48, 4
    Q, K, V = gen.random_qkv(1, 1, N, 128, seed=48)
    v = rng.random((1, N)).astype(np.float32)
    s = rng.random((1, N)).astype(np.float32)
    # block size 1: a block pair is an element pair, the two forms give the same attention output
    blk = np.zeros((1, N, N), np.float32)
    a = orc.build_index(v, s, blk, N, 1, w, _bud(k_slash=5, k_blocks=N), override=[IS])
    c = orc.build_index(v, s, blk, N, 1, w, _bud(k_slash=5, k_blocks=N, diagonal_select=1), override=[IS])
    Oa, _, ka = orc.masked_rows(Q, K, V, 1, a)
    Oc, _, kc = orc.masked_rows(Q, K, V, 1, c)
    assert (ka == kc).all() and np.abs(Oa - Oc).max() < 1e-12
    # only offset 0 selected: nothing beyond the diagonal blocks
    s0 = np.zeros((1, N), np.float32); s0[0, 0] = 1.0
    blk = np.zeros((1, 6, 6), np.float32)
    c = orc.build_index(v, s0, blk, N, 8, w, _bud(k_slash=1, k_blocks=6, diagonal_select=1), override=[IS])
    assert _csr_pairs(c, 0, 6) == {(R, R) for R in range(6)}
    # offset b: exactly the block below the diagonal; offset b + 1: the two blocks below it
    for o, want_extra in ((8, {(R, R - 1) for R in range(1, 6)}),
                          (9, {(R, R - 1) for R in range(1, 6)} | {(R, R - 2) for R in range(2, 6)})):
        so = np.zeros((1, N), np.float32); so[0, o] = 1.0
        c = orc.build_index(v, so, blk, N, 8, w, _bud(k_slash=1, k_blocks=6, diagonal_select=1), override=[IS])
        assert _csr_pairs(c, 0, 6) == {(R, R) for R in range(6)} | want_extra
    # the other patterns ignore the setting
    for pat in (T, BC):
        a = orc.build_index(v, s, blk, N, 8, w, _bud(k_blocks=9), override=[pat])
        c = orc.build_index(v, s, blk, N, 8, w, _bud(k_blocks=9, diagonal_select=1), override=[pat])
        assert all(x.tobytes() == y.tobytes() for x, y in zip(a.arrays()[:6], c.arrays()[:6]))


@settings(max_examples=30, deadline=None)
@given(st.lists(st.integers(0, 6), min_size=36, max_size=36), st.integers(6, 21), st.integers(0, 3))
def test_row_normalised_block_key_is_the_global_rule_on_the_scaled_map(vals, kb, seed):
    # block_select 2 must select what the (already pinned) global rule selects on blk[R][C] * (R+1),
    # the scaling done here in numpy float32
    nb, b = 6, 4
    N = nb * b
    rng = np.random.default_rng(seed)
    blk = (np.array(vals, np.float32).reshape(1, nb, nb) * np.float32(0.125)
           + rng.random((1, nb, nb)).astype(np.float32) * np.float32(seed > 0))
    v = np.ones((1, N), np.float32)
    scaled = (blk * np.arange(1, nb + 1, dtype=np.float32)[None, :, None]).astype(np.float32)
    a = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=kb, block_select=2), override=[BC])
    c = orc.build_index(v, v, scaled, N, b, 4, _bud(k_blocks=kb, block_select=0), override=[BC])
    assert all(x.tobytes() == y.tobytes() for x, y in zip(a.arrays(), c.arrays()))


def test_row_normalised_block_key_prefers_relative_peaks():
    # a block that is 3x its row's uniform value in a long row against one that is 1.5x in a short
    # row: the raw rule takes the short row's (larger absolute value), the normalised one the other
    nb, b = 8, 4
    N = nb * b
    blk = np.zeros((1, nb, nb), np.float32)
    for R in range(nb):
        blk[0, R, :R + 1] = 1.0 / (R + 1)
    blk[0, 1, 0] = 1.5 / 2          # 0.75
    blk[0, 7, 2] = 3.0 / 8          # 0.375
    v = np.ones((1, N), np.float32)
    raw = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=nb + 1, block_select=0), override=[BC])
    nrm = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=nb + 1, block_select=2), override=[BC])
    assert _csr_pairs(raw, 0, nb) - {(R, R) for R in range(nb)} == {(1, 0)}
    assert _csr_pairs(nrm, 0, nb) - {(R, R) for R in range(nb)} == {(7, 2)}


def test_k_larger_than_candidates_is_clamped():
    N, b = 16, 4
    v = np.arange(16, dtype=np.float32)[None]
    blk = np.random.default_rng(0).random((1, 4, 4)).astype(np.float32)
    ix = orc.build_index(v, v, blk, N, b, 4, _bud(k_vertical=20, k_slash=18, k_blocks=30),
                         override=[IS])
    assert ix.n_cols[0] == 16 and (ix.cols[0, :16] == np.arange(16)).all() and (ix.cols[0, 16:] == -1).all()
    assert ix.n_offs[0] == 16
    ix = orc.build_index(v, v, blk, N, b, 4, _bud(k_blocks=30), override=[BC])
    assert ix.rowptr[0, -1] == 10                 # all causal blocks


def test_triangular_csr_matches_definition():
    N, b = 40 * 8, 8
    nb = N // b
    v = np.ones((1, N), np.float32)
    bud = _bud(sink_blocks=2, local_blocks=5, k_blocks=10)
    ix = orc.build_index(v, v, np.zeros((1, nb, nb), np.float32), N, b, 8, bud, override=[T])
    R, C = np.tril_indices(nb)
    keep = (C < 2) | (R - C < 5)
    assert ix.rowptr[0, -1] == keep.sum() == orc.triangular_count(nb, 2, 5)
    got = [(r, int(c)) for r in range(nb) for c in ix.blkcols[0, ix.rowptr[0, r]:ix.rowptr[0, r + 1]]]
    assert got == sorted(zip(R[keep].tolist(), C[keep].tolist()))
    assert ix.n_cols[0] == 0 and ix.n_offs[0] == 0 and (ix.cols == -1).all()


# ---- default budgets: the values of the benchmark definition's five shapes

def _golden_budgets():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "default_budgets.txt")
    rows = []
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            rows.append((int(f[0]), int(f[1]), float(f[2]), tuple(int(x) for x in f[3:7])))
    assert len(rows) == 5
    return rows


@pytest.mark.parametrize("N,b,rho,want", _golden_budgets())
def test_default_budgets_table(N, b, rho, want):
    bud = orc.default_budgets(N, b, rho)
    assert (bud.k_blocks, bud.local_blocks, bud.k_vertical, bud.k_slash) == want
    nb = N // b
    # L is the largest band that fits: the real block count fits, one more does not
    assert orc.triangular_count(nb, bud.sink_blocks, bud.local_blocks) <= bud.k_blocks
    L1 = bud.local_blocks + 1
    assert L1 * nb - L1 * (L1 - 1) // 2 + (nb - L1) * bud.sink_blocks > bud.k_blocks


# ---- pattern rule: decided cases and the exact boundary

def _fx(x):
    return int(np.floor(float(np.float32(x)) * 2.0 ** 30))


def _rule_bigint(v, s, N, b, w, bud):
    nb = N // b
    sb = min(bud.sink_blocks * b, N)
    lb0 = max((nb - bud.local_blocks) * b, sb)
    Vtot = sum(_fx(x) for x in v)
    CT = sum(_fx(x) for j, x in enumerate(v) if j < sb or j >= lb0)
    E = sum(N - w + i + 1 for i in range(w))
    ET = sum(min(sb, N - w + i + 1) + max(0, N - w + i + 1 - lb0) for i in range(w))
    if bud.lift_den * CT * E >= bud.lift_num * Vtot * ET:
        return T
    top = lambda a, k: sum(sorted((_fx(x) for x in a), reverse=True)[:k])
    if bud.lift_den * (top(v, bud.probe_v) + top(s, bud.probe_s)) * E >= \
            bud.lift_num * Vtot * (bud.probe_v + bud.probe_s) * w:
        return IS
    return BC


def test_pattern_rule_decided_cases():
    N, b, w = 1024, 64, 64
    bud = _bud(sink_blocks=1, local_blocks=2)
    inv = 1.0 / (np.arange(N - w, N) + 1.0)
    uni = np.array([inv[max(0, j - (N - w)):].sum() for j in range(N)], np.float32)
    assert orc.choose_pattern(uni, uni, N, b, w, bud) == BC          # uniform head: lift 1
    tri = np.zeros(N, np.float32); tri[:4] = 8.0; tri[N - 128:] = 0.25
    assert orc.choose_pattern(tri, uni, N, b, w, bud) == T
    col = uni.copy(); col[[100, 300, 500, 700]] = 6.0                 # four heavy columns, mid-sequence
    assert orc.choose_pattern(col, uni, N, b, w, bud) == IS
    sl = uni.copy(); sl[[7, 200]] = 20.0                              # two heavy diagonals
    assert orc.choose_pattern(uni, sl, N, b, w, bud) == IS


def test_pattern_rule_exact_boundary():
    # choose masses so that lift_den*C_T*E == lift_num*Vtot*E_T exactly, then nudge one ulp
    N, b, w = 256, 64, 64
    bud = _bud(sink_blocks=1, local_blocks=1, lift_num=2, lift_den=1)
    E = sum(N - w + i + 1 for i in range(w))
    ET = sum(min(64, N - w + i + 1) + max(0, N - w + i + 1 - 192) for i in range(w))
    # v: x on the 128 region keys, y elsewhere; need C_T*E == 2*Vtot*E_T
    # C_T = 128x, Vtot = 128x + 128y  ->  x*(E - 2*ET) = 2*ET*y
    x, y = 2 * ET, E - 2 * ET
    scale = 2.0 ** -14
    v = np.full(N, y * scale, np.float32); v[:64] = x * scale; v[192:] = x * scale
    assert float(v[0]) == x * scale and float(v[100]) == y * scale
    s = np.zeros(N, np.float32)
    assert _rule_bigint(v, s, N, b, w, bud) == T
    assert orc.choose_pattern(v, s, N, b, w, bud) == T                # equality counts as Triangular
    v2 = v.copy(); v2[100] = np.nextafter(v2[100], np.float32(np.inf))
    assert _rule_bigint(v2, s, N, b, w, bud) != T
    assert orc.choose_pattern(v2, s, N, b, w, bud) == _rule_bigint(v2, s, N, b, w, bud)


@settings(max_examples=30, deadline=None)
@given(st.integers(0, 2 ** 31 - 1))
def test_pattern_rule_matches_bigint(seed):
    rng = np.random.default_rng(seed)
    N, b, w = 128, 16, 16
    v = (rng.random(N) ** 8 * 16).astype(np.float32)
    s = (rng.random(N) ** 8 * 16).astype(np.float32)
    bud = _bud(sink_blocks=1, local_blocks=int(rng.integers(1, 4)), lift_num=int(rng.integers(1, 6)))
    assert orc.choose_pattern(v, s, N, b, w, bud) == _rule_bigint(v, s, N, b, w, bud)


# ---- planted recovery: with k = planted counts the selected sets are the planted sets

def _recover(wl):
    data = gen.generate(wl)
    N, b, w = wl.seq_len, wl.block, wl.last_q
    v, s, blk = orc.estimate(data["Q"], data["K"], b, w)
    return data, v.astype(np.float32), s.astype(np.float32), blk.astype(np.float32)


def test_planted_recovery_cfg1():
    wl = gen.WORKLOADS["cfg1"]
    data, v, s, blk = _recover(wl)
    bud = orc.default_budgets(wl.seq_len, wl.block, wl.keep)
    bud.k_vertical, bud.k_slash = 4, 3
    ix = orc.build_index(v, s, blk, wl.seq_len, wl.block, wl.last_q, bud,
                         override=[IS] * wl.n_q_heads)
    for h in range(wl.n_q_heads):
        assert ix.cols[h].tolist() == [0, 1, 2, 3]
        assert ix.offs[h].tolist() == [0, 64, 512]


def test_planted_recovery_small_mixed():
    # +3 logit plants against lognormal noise: a planted item always ranks inside the
    # best 2k, and the hot blocks are inside the default block budget
    # (one global top-k over raw block softmax values fills short early rows first)
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="mini3", n_q_heads=8, n_kv_heads=2,
                    seq_len=8192, seed=77, n_hot=12, keep=0.25)
    data, v, s, blk = _recover(wl)
    N, b, w = wl.seq_len, wl.block, wl.last_q
    bud = orc.default_budgets(N, b, wl.keep)
    bud.k_vertical, bud.k_slash = 2 * wl.n_cols, 2 * wl.n_offs
    planted = [p.pattern for p in data["plants"]]
    ix = orc.build_index(v, s, blk, N, b, w, bud, override=planted)
    for h, p in enumerate(data["plants"]):
        if p.pattern == IS:
            assert set(p.cols.tolist()) <= set(ix.cols[h].tolist())
            assert set(p.offs.tolist()) <= set(ix.offs[h].tolist())
        if p.pattern == BC:
            got = {(R, int(C)) for R in range(N // b)
                   for C in ix.blkcols[h, ix.rowptr[h, R]:ix.rowptr[h, R + 1]] if C != R}
            assert {(int(R), int(C)) for R, C in p.hot} <= got
            assert len(got) == bud.k_blocks - N // b
    # the run-time rule agrees with the plant on Triangular / Interval-Slash heads
    auto = orc.build_index(v, s, blk, N, b, w, orc.default_budgets(N, b, wl.keep)).pattern
    for h, p in enumerate(data["plants"]):
        if p.pattern in (T, IS):
            assert auto[h] == p.pattern


@pytest.mark.parametrize("N,b,bud", [
    (1024, 64, orc.Budgets(1, 3, 40, 4, 30)),
    (1024, 64, orc.Budgets(2, 16, 40, 4, 16)),                      # band = everything: the Triangular count rules
    (2048, 128, orc.Budgets(1, 2, 64, 6, 60, block_select=1)),      # per-row shares round up
    (1024, 64, orc.Budgets(1, 2, 40, 5, 20, diagonal_select=1)),    # widened diagonals: two key blocks per offset
    (1024, 64, orc.Budgets(0, 1, 40, 1024, 16, diagonal_select=1)), # every offset selected
])
def test_block_capacity_bounds_every_index_the_oracle_builds(N, b, bud):
    # block_capacity is a buffer size; it is pinned against the blocks counted in indices the oracle
    # itself builds under every override, and against the Triangular set written out with numpy
    nb, w, H = N // b, 32, 3
    cap = orc.block_capacity(N, b, bud)
    R, Cc = np.arange(nb)[:, None], np.arange(nb)[None, :]
    tri = int(((Cc <= R) & ((Cc < bud.sink_blocks) | (R - Cc < bud.local_blocks))).sum())
    assert cap >= tri
    rng = np.random.default_rng(5)
    seen = 0
    for trial in range(4):
        v = rng.random((H, N), dtype=np.float32)
        s = rng.random((H, N), dtype=np.float32)
        blk = np.tril(rng.random((H, nb, nb), dtype=np.float32))
        if trial == 1:    # offsets spread so that widened diagonals touch as many distinct blocks as they can
            s[:] = 0
            s[:, (np.arange(N) % b) == b // 2] = 1
        for pat in (0, 1, 2):
            ix = orc.build_index(v, s, blk, N, b, w, bud, override=[pat] * H)
            cnt = ix.rowptr[:, nb]
            assert (cnt <= cap).all(), (pat, cnt, cap)
            assert ((ix.blkcols >= 0).sum(1) == cnt).all()
            if pat == 0:
                assert (cnt == tri).all()
            seen = max(seen, int(cnt.max()))
    if not bud.diagonal_select and bud.block_select != 1:
        assert seen == cap            # tight: some pattern fills the buffer
    elif bud.block_select == 1:       # per-row shares: each of the nb rows rounds up by less than one block
        assert bud.k_blocks <= seen <= cap and cap - bud.k_blocks <= nb
