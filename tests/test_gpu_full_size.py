"""Whole path at the benchmark's sizes, in the launch configuration bench.py times:
scores by tolerance, index bit-exact on the GPU's own scores, attention on sampled rows."""
import numpy as np
import pytest
import torch

from harness import gen
from oracle import oracle as orc
from gpu_util import (assert_index_equal, check_attention, dev_bf16, download_index,
                      download_scores, host_f64)
import paper_2412_06198_amd as sa

pytestmark = pytest.mark.gpu


SENTINEL = 30000.0      # no attention output comes near it: |O| is bounded by max |V| (a few units)


def _item_rows(rng, N, extra):
    """One row in every 128-row work item of the attention kernel (the same rows for every head, so
    every (head, item) pair is sampled), plus `extra` random rows and the first / middle / last."""
    starts = np.arange(0, N, 128)
    per_item = starts + rng.integers(0, np.minimum(128, N - starts))
    rows = np.concatenate([per_item, rng.choice(N, extra, replace=False), [0, N // 2 + 1, N - 1]])
    return np.unique(rows).astype(np.int32)


def _check_prefill(ses, data, b, got, Q, K, V, rows, what):
    """sa_sparse_prefill on the index the session holds: every output element is written (O starts
    as a sentinel no result can equal) and the sampled rows match the oracle on that index."""
    O = torch.full_like(Q, SENTINEL)
    ses.prefill(Q, K, V, O)
    torch.cuda.synchronize()
    assert bool((O.float().abs() < 1e3).all()), f"{what}: some output rows were never written"
    ref, ws, _ = orc.masked_rows(data["Q"], data["K"], data["V"], b, got, rows=rows)
    assert np.abs(ws - 1).max() < 1e-9
    check_attention(host_f64(O[:, torch.from_numpy(rows.astype(np.int64)).cuda()]), ref, what)
    return O


def _whole_path(name, n_rows, margin_check=True, wl=None, twice=False):
    print(f"case full-size {name}", flush=True)
    wl = gen.WORKLOADS[name] if wl is None else wl
    data = gen.generate(wl)
    N, b, w, Hq = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads
    ses = sa.Session(Hq, wl.n_kv_heads, N, b, w, keep=wl.keep)
    Q, K, V = dev_bf16(data["Q"]), dev_bf16(data["K"]), dev_bf16(data["V"])
    ses.estimate(Q, K)
    ses.build_index(None)
    v, s, blk = download_scores(ses)
    got = download_index(ses)
    print("  gpu done; oracle estimate", flush=True)
    # 1. scores
    rv, rs, rblk = orc.estimate(data["Q"], data["K"], b, w)
    for nm, g_, r_ in (("v", v, rv), ("s", s, rs), ("blk", blk, rblk)):
        bad = np.abs(g_ - r_) > 1e-3 * np.abs(r_) + 1e-6 * w
        assert not bad.any(), (nm, int(bad.sum()))
    # 2. selection: bit-exact on the GPU's own fp32 scores
    bud = orc.default_budgets(N, b, wl.keep)
    want = orc.build_index(v, s, blk, N, b, w, bud)
    assert_index_equal(got, want)
    # 3. end to end: heads whose pattern decision and top-k boundaries are not near-ties in
    #    fp64 must give the same index from the oracle's own scores
    e2e = orc.build_index(rv.astype(np.float32), rs.astype(np.float32), rblk.astype(np.float32),
                          N, b, w, bud)
    same = [h for h in range(Hq) if all(a[h].tobytes() == c[h].tobytes()
                                        for a, c in zip(got.arrays(), e2e.arrays()))]
    print(f"  end-to-end identical heads: {len(same)}/{Hq}; patterns {got.pattern.tolist()}", flush=True)
    assert (got.pattern == e2e.pattern).all()
    for h in range(Hq):
        if h in same:
            continue
        # differing heads may only differ by candidates whose fp64 scores tie within 1e-3
        for arr_g, arr_o, sc in ((got.cols[h], e2e.cols[h], rv[h]), (got.offs[h], e2e.offs[h], rs[h])):
            a, c = set(arr_g[arr_g >= 0].tolist()), set(arr_o[arr_o >= 0].tolist())
            if a != c:
                lo = min(sc[list(a | c)])
                for j in a ^ c:
                    assert abs(sc[j] - lo) <= 2e-3 * lo, (h, j)
    # 4. attention, oracle evaluated on the GPU's index: a row of every 128-row item of every head
    #    plus random rows; every element of O written
    rng = np.random.Generator(np.random.Philox(key=[wl.seed, 5]))
    rows = _item_rows(rng, N, n_rows)
    print(f"  oracle attention on {rows.size} rows per head", flush=True)
    O = _check_prefill(ses, data, b, got, Q, K, V, rows, name)
    if twice:
        # the same inputs give the same bytes, run to run: scores, index and output
        ses.estimate(Q, K)
        ses.build_index(None)
        O2 = torch.full_like(Q, SENTINEL)
        ses.prefill(Q, K, V, O2)
        for a, c in zip(download_scores(ses), (v, s, blk)):
            assert a.tobytes() == c.tobytes()
        assert_index_equal(download_index(ses), got)
        assert torch.equal(O, O2)
    return ses, (Q, K, V, O), got, data


def test_cfg2_16k():
    _whole_path("cfg2", 96)


def test_cfg3_32k():
    _whole_path("cfg3", 96)


def test_cfg4_64k():
    _whole_path("cfg4", 64)


def test_cfg5_128k_one_layer():
    _whole_path("cfg5", 48, twice=True)


@pytest.mark.parametrize("forced", [orc.INTERVAL_SLASH, orc.TRIANGULAR])
def test_cfg5_128k_every_head_one_pattern(forced):
    # 8 KV heads at 128K: two work queues share a KV head (the queue mapping that only this size
    # reaches), and with every head Interval-Slash every item runs the diagonal phase.  Index
    # byte-identical to the oracle under the override, attention on a row of every item of every head.
    print(f"case cfg5 forced pattern {forced}", flush=True)
    wl = gen.WORKLOADS["cfg5"]
    data = gen.generate(wl)
    N, b, w, Hq = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads
    ses = sa.Session(Hq, wl.n_kv_heads, N, b, w, keep=wl.keep)
    Q, K, V = dev_bf16(data["Q"]), dev_bf16(data["K"]), dev_bf16(data["V"])
    ses.estimate(Q, K)
    ses.build_index([forced] * Hq)
    v, s, blk = download_scores(ses)
    got = download_index(ses)
    want = orc.build_index(v, s, blk, N, b, w, orc.default_budgets(N, b, wl.keep), override=[forced] * Hq)
    assert_index_equal(got, want)
    assert (got.pattern == forced).all()
    rng = np.random.Generator(np.random.Philox(key=[wl.seed, 6 + forced]))
    _check_prefill(ses, data, b, got, Q, K, V, _item_rows(rng, N, 16), f"cfg5 forced {forced}")


def test_ragged_33k_whole_path():
    # 521 blocks of 64: the last 1024-key chunk of the estimator, the last 128-row item of the
    # attention kernel and the last 16-row strip of the block map are all partial
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="ragged33k", seq_len=521 * 64, block=64, n_q_heads=8,
                    n_kv_heads=2, keep=0.06, hot_block=64, seed=9100)
    _whole_path("ragged33k", 64, wl=wl)


def test_longest_supported_sequence_256k():
    # the library's limit: 262144 tokens, block 64 (4096 key tiles, the widest tile-list entries),
    # one KV head (all eight work queues on one head), one head per pattern
    wl = gen.scaled(gen.WORKLOADS["cfg5"], name="max256k", seq_len=262144, block=64, n_q_heads=4,
                    n_kv_heads=1, keep=0.01, hot_block=64, seed=9000)
    _whole_path("max256k", 40, wl=wl)


def test_cfg5_one_call_estimate_and_index():
    # the launch configuration bench.py times: scores and index of the one-call form against the
    # two calls, byte for byte, at the benchmark size
    print("case cfg5 one-call", flush=True)
    wl = gen.WORKLOADS["cfg5"]
    data = gen.generate(wl)
    N, b, w, Hq = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads
    Q, K = dev_bf16(data["Q"]), dev_bf16(data["K"])
    two = sa.Session(Hq, wl.n_kv_heads, N, b, w, keep=wl.keep)
    one = sa.Session(Hq, wl.n_kv_heads, N, b, w, keep=wl.keep)
    two.estimate(Q, K)
    two.build_index(None)
    for rep in range(3):
        one.estimate_and_index(Q, K, None)
        for a, c in zip(download_scores(two), download_scores(one)):
            assert a.tobytes() == c.tobytes()
        assert_index_equal(download_index(one), download_index(two))
    assert len(set(download_index(one).pattern.tolist())) == 3
    # the same with the block map computed for the Block-Cluster heads only
    lazy = sa.Session(Hq, wl.n_kv_heads, N, b, w, keep=wl.keep, lazy_block_map=1)
    lazy.blk.fill_(-7)
    for rep in range(2):
        lazy.estimate_and_index(Q, K, None)
        want = download_index(two)
        assert_index_equal(download_index(lazy), want)
        assert torch.equal(lazy.v, two.v) and torch.equal(lazy.s, two.s)
        bc = torch.from_numpy(want.pattern == 2).cuda()
        assert torch.equal(lazy.blk[bc], two.blk[bc])
        assert bool((lazy.blk[~bc] == -7).all())


def test_counters_match_oracle_mask_count():
    print("case counters", flush=True)
    Hq, Hkv, N, b, w = 4, 2, 1024, 64, 64
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=3)
    bud = orc.Budgets(1, 2, 40, 3, N // b + 20)
    ses = sa.Session(Hq, Hkv, N, b, w, sink_blocks=1, local_blocks=2, k_vertical=40, k_slash=3,
                     k_blocks=N // b + 20)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    O = torch.empty_like(Qd)
    ses.estimate(Qd, Kd)
    ses.build_index([0, 1, 2, 1])
    tiles, kept = ses.prefill_counted(Qd, Kd, Vd, O)
    ix = download_index(ses)
    assert kept == sum(orc.mask_count(N, b, h, ix) for h in range(Hq))
    assert tiles * 32 * 32 >= kept
    O2 = torch.empty_like(Qd)
    ses.prefill(Qd, Kd, Vd, O2)
    torch.cuda.synchronize()
    assert torch.equal(O, O2)


def test_decode_step_at_cfg5_128k():
    # the decode step at the benchmark's size and launch configuration (bench.py --decode):
    # every head against the fp64 oracle, run-time patterns, a position behind a few generated keys
    from oracle import decode as dec
    print("case decode cfg5", flush=True)
    wl = gen.WORKLOADS["cfg5"]
    data = gen.generate(wl)
    Hq, Hkv, N, b, d = wl.n_q_heads, wl.n_kv_heads, wl.seq_len, wl.block, wl.head_dim
    pad = 64
    Kx = np.concatenate([data["K"], data["K"][:, :pad]], axis=1)
    Vx = np.concatenate([data["V"], data["V"][:, :pad]], axis=1)
    ses = sa.Session(Hq, Hkv, N, b, wl.last_q, keep=wl.keep, kv_head_stride=(N + pad) * d)
    Qd, Kd, Vd = dev_bf16(data["Q"]), dev_bf16(Kx), dev_bf16(Vx)
    ses.estimate(Qd, Kd)
    ses.build_index(None)
    torch.cuda.synchronize()
    ix = download_index(ses)
    pos = N + 7
    q = Qd[:, N - 1].contiguous()
    o = torch.empty_like(q)
    ses.decode(q, Kd, Vd, pos, o)
    torch.cuda.synchronize()
    ref, cnt = dec.decode_step(data["Q"][:, N - 1], Kx, Vx, b, ix, N, pos)
    err = np.abs(host_f64(o) - ref)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3, (float(err.max()), float(err.mean()))
    assert (cnt >= pos - N + 1).all()
