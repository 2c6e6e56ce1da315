"""GPU parity of sa_estimate_patterns (tolerance) and sa_build_index (bit-exact)."""
import numpy as np
import pytest
import torch

from harness import gen
from oracle import oracle as orc
from gpu_util import (assert_index_equal, dev_bf16, download_index, download_scores,
                      make_session, upload_scores)

pytestmark = pytest.mark.gpu
T, IS, BC = 0, 1, 2


def _check_scores(got, ref, w):
    for name, g, r in zip("v s blk".split(), got, ref):
        tol = 1e-3 * np.abs(r) + 1e-6 * w
        bad = np.abs(g.astype(np.float64) - r) > tol
        assert not bad.any(), (name, int(bad.sum()), float(np.abs(g - r).max()))


@pytest.mark.parametrize("Hq,Hkv,N,b,w", [(4, 2, 1024, 64, 64), (4, 4, 768, 128, 64),
                                          (8, 2, 2048 + 64, 64, 17), (2, 2, 64, 64, 64),
                                          (6, 1, 512, 128, 33), (4, 2, 273 * 64, 64, 64),
                                          (4, 2, 521 * 64, 64, 64), (2, 1, 261 * 128, 128, 40)])
def test_scores_match_oracle(Hq, Hkv, N, b, w):
    print(f"case scores Hq={Hq} Hkv={Hkv} N={N} b={b} w={w}", flush=True)
    Q, K, _ = gen.random_qkv(Hq, Hkv, N, 128, seed=N + w)
    ses = make_session(Hq, Hkv, N, b, w, orc.default_budgets(N, b, 0.5))
    ses.estimate(dev_bf16(Q), dev_bf16(K))
    got = download_scores(ses)
    _check_scores(got, orc.estimate(Q, K, b, w), w)
    ses.estimate(dev_bf16(Q), dev_bf16(K))
    again = download_scores(ses)
    for a, c in zip(got, again):
        assert a.tobytes() == c.tobytes()          # deterministic


@pytest.mark.parametrize("N,b,keep", [(4096, 64, 0.10), (2048, 128, 0.3)])
def test_index_bit_exact_on_gpu_scores(N, b, keep):
    print(f"case index N={N} b={b}", flush=True)
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=8, n_kv_heads=2, seq_len=N,
                    block=b, seed=N, n_hot=8, hot_block=b, keep=keep)
    data = gen.generate(wl)
    bud = orc.default_budgets(N, b, keep)
    ses = make_session(8, 2, N, b, 64, bud)
    ses.estimate(dev_bf16(data["Q"]), dev_bf16(data["K"]))
    v, s, blk = download_scores(ses)
    for ov in (None, [T, IS, BC, IS, BC, T, IS, BC], [BC] * 8, [IS] * 8):
        ses.build_index(ov)
        got = download_index(ses)
        want = orc.build_index(v, s, blk, N, b, 64, bud, override=ov)
        assert_index_equal(got, want)


def test_index_ties_bit_exact():
    # small-integer scores: most candidates tie at the selection boundary
    print("case ties", flush=True)
    Hq, N, b, w = 4, 1024, 64, 64
    nb = N // b
    rng = np.random.default_rng(5)
    v = rng.integers(0, 4, (Hq, N)).astype(np.float32)
    s = rng.integers(0, 3, (Hq, N)).astype(np.float32)
    blk = np.tril(rng.integers(0, 5, (Hq, nb, nb))).astype(np.float32) * 0.25
    for kv, ks, kb in [(100, 7, nb + 40), (N, N, nb * (nb + 1) // 2), (1, 1, nb), (513, 300, nb + 1)]:
        bud = orc.Budgets(1, 2, kv, ks, kb)
        ses = make_session(Hq, 2, N, b, w, bud)
        upload_scores(ses, v, s, blk)
        for ov in ([IS] * Hq, [BC] * Hq, [T] * Hq, None):
            ses.build_index(ov)
            assert_index_equal(download_index(ses), orc.build_index(v, s, blk, N, b, w, bud, override=ov))


def test_pattern_rule_boundary_on_gpu():
    # the exact-equality case of the Triangular test and its one-ulp neighbour
    print("case rule boundary", flush=True)
    N, b, w = 256, 64, 64
    bud = orc.Budgets(1, 1, 4, 4, 4, lift_num=2, lift_den=1)
    E = sum(N - w + i + 1 for i in range(w))
    ET = sum(min(64, N - w + i + 1) + max(0, N - w + i + 1 - 192) for i in range(w))
    x, y, sc = 2 * ET, E - 2 * ET, 2.0 ** -14
    v = np.full((2, N), y * sc, np.float32)
    v[:, :64] = x * sc
    v[:, 192:] = x * sc
    v[1, 100] = np.nextafter(v[1, 100], np.float32(np.inf))
    s = np.zeros((2, N), np.float32)
    blk = np.zeros((2, 4, 4), np.float32)
    ses = make_session(2, 2, N, b, w, bud)
    upload_scores(ses, v, s, blk)
    ses.build_index(None)
    got = download_index(ses)
    want = orc.build_index(v, s, blk, N, b, w, bud)
    assert got.pattern[0] == T and got.pattern[1] != T
    assert_index_equal(got, want)


@pytest.mark.parametrize("N,b,keep,rows", [(4096, 64, 0.10, 0), (2048, 128, 0.3, 1), (8192 + 128, 128, 0.07, 0),
                                           (1024, 64, 0.5, 1)])
def test_one_call_estimate_and_index_is_byte_identical(N, b, keep, rows):
    # sa_estimate_and_index against sa_estimate_patterns + sa_build_index: same scores, same index
    print(f"case one-call N={N} b={b} rows={rows}", flush=True)
    Hq, Hkv = 8, 2
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=Hq, n_kv_heads=Hkv, seq_len=N,
                    block=b, seed=N + 3, n_hot=4, hot_block=b, keep=keep)
    data = gen.generate(wl)
    bud = orc.default_budgets(N, b, keep)
    bud.block_select = rows
    Q, K = dev_bf16(data["Q"]), dev_bf16(data["K"])
    two, one = make_session(Hq, Hkv, N, b, 64, bud), make_session(Hq, Hkv, N, b, 64, bud)
    for ov in (None, [T, IS, BC, IS, BC, T, IS, BC], [BC] * Hq, None):
        two.estimate(Q, K)
        two.build_index(ov)
        for t in one.index_tensors() + [one.v, one.s, one.blk]:
            t.fill_(-7)                      # stale contents must not survive
        one.estimate_and_index(Q, K, ov)
        for a, c in zip(download_scores(two), download_scores(one)):
            assert a.tobytes() == c.tobytes()
        want = download_index(two)
        assert_index_equal(download_index(one), want)
    v, s, blk = download_scores(one)
    assert_index_equal(download_index(one), orc.build_index(v, s, blk, N, b, 64, bud))


@pytest.mark.gpu
@pytest.mark.parametrize("N,b,keep,rows,diag", [(4096, 64, 0.10, 0, 0), (2048, 128, 0.3, 1, 0),
                                                (8192 + 128, 128, 0.07, 2, 1), (1024, 64, 0.5, 0, 0)])
def test_lazy_block_map_gives_the_same_index(N, b, keep, rows, diag):
    # lazy_block_map: the block map exists for the Block-Cluster heads only; v, s and the index are
    # those of the two calls, byte for byte, and the block map of the other heads is not written
    print(f"case lazy N={N} b={b} rows={rows} diag={diag}", flush=True)
    Hq, Hkv = 8, 2
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=Hq, n_kv_heads=Hkv, seq_len=N,
                    block=b, seed=N + 5, n_hot=4, hot_block=b, keep=keep)
    data = gen.generate(wl)
    bud = orc.default_budgets(N, b, keep)
    bud.block_select, bud.diagonal_select = rows, diag
    Q, K = dev_bf16(data["Q"]), dev_bf16(data["K"])
    two, lazy = make_session(Hq, Hkv, N, b, 64, bud), make_session(Hq, Hkv, N, b, 64, bud, lazy_block_map=1)
    seen = set()
    for ov in (None, [T, IS, BC, IS, BC, T, IS, BC], [BC] * Hq, [T] * Hq, None):
        two.estimate(Q, K)
        two.build_index(ov)
        for t in lazy.index_tensors() + [lazy.v, lazy.s, lazy.blk]:
            t.fill_(-7)
        lazy.estimate_and_index(Q, K, ov)
        want = download_index(two)
        assert_index_equal(download_index(lazy), want)
        v2, s2, blk2 = download_scores(two)
        v1, s1, blk1 = download_scores(lazy)
        assert v1.tobytes() == v2.tobytes() and s1.tobytes() == s2.tobytes()
        for h in range(Hq):
            seen.add(int(want.pattern[h]))
            if want.pattern[h] == BC:
                assert blk1[h].tobytes() == blk2[h].tobytes(), h
            else:
                assert (blk1[h] == -7).all(), h
    assert seen == {T, IS, BC}
    # the separate calls of a lazy context still compute every head's block map
    lazy.blk.fill_(-7)
    lazy.estimate(Q, K)
    lazy.build_index(None)
    assert download_scores(lazy)[2].tobytes() == blk2.tobytes()
    assert_index_equal(download_index(lazy), want)
