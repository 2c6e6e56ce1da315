"""GPU parity of block-granular diagonals (an Interval-Slash head keeps every block pair that holds
a pair of a selected diagonal): index bit-exact, attention within the usual tolerance."""
import dataclasses

import numpy as np
import pytest
import torch

from harness import gen
from oracle import oracle as orc
from gpu_util import (assert_index_equal, check_attention, dev_bf16, download_index,
                      download_scores, host_f64, make_session, upload_scores)

pytestmark = pytest.mark.gpu
T, IS, BC = 0, 1, 2


@pytest.mark.parametrize("N,b,keep,rows", [(4096, 64, 0.10, 0), (2048, 128, 0.3, 1), (8192 + 128, 128, 0.07, 0)])
def test_diag_blocks_index_bit_exact_on_gpu_scores(N, b, keep, rows):
    print(f"case diag-blocks index N={N} b={b} rows={rows}", flush=True)
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=8, n_kv_heads=2, seq_len=N,
                    block=b, seed=N + 2, n_hot=8, hot_block=b, keep=keep)
    data = gen.generate(wl)
    bud = dataclasses.replace(orc.default_budgets(N, b, keep), diagonal_select=1, block_select=rows)
    ses = make_session(8, 2, N, b, 64, bud)
    Q, K = dev_bf16(data["Q"]), dev_bf16(data["K"])
    ses.estimate(Q, K)
    v, s, blk = download_scores(ses)
    for ov in (None, [T, IS, BC, IS, BC, T, IS, BC], [IS] * 8):
        ses.build_index(ov)
        got = download_index(ses)
        assert_index_equal(got, orc.build_index(v, s, blk, N, b, 64, bud, override=ov))
        assert (got.n_offs == 0).all()
    ses.estimate_and_index(Q, K, [IS] * 8)           # the one-call form takes the same path
    assert_index_equal(download_index(ses), got)


def test_diag_blocks_ties_and_limits():
    # heavy ties among the diagonal scores; from one offset to every offset (all causal blocks)
    print("case diag-blocks ties", flush=True)
    Hq, N, b, w = 4, 1024, 64, 64
    nb = N // b
    rng = np.random.default_rng(8)
    v = rng.integers(0, 4, (Hq, N)).astype(np.float32)
    s = rng.integers(0, 3, (Hq, N)).astype(np.float32)
    s[2] = 0.0
    s[2, [0, 63, 64, 65, 1023]] = [5, 4, 3, 2, 1]      # block-boundary offsets and the longest one
    blk = np.tril(rng.random((Hq, nb, nb))).astype(np.float32)
    for ks in (1, 2, 5, 40, 300, N):
        bud = orc.Budgets(1, 2, 16, ks, nb + 8, diagonal_select=1)
        ses = make_session(Hq, 2, N, b, w, bud)
        upload_scores(ses, v, s, blk)
        for ov in ([IS] * Hq, [T, BC, IS, IS], None):
            ses.build_index(ov)
            got = download_index(ses)
            assert_index_equal(got, orc.build_index(v, s, blk, N, b, w, bud, override=ov))
            if ks == N and ov == [IS] * Hq:
                assert (got.rowptr[:, nb] == nb * (nb + 1) // 2).all()


def test_diag_blocks_attention_matches_oracle():
    print("case diag-blocks attention", flush=True)
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=8, n_kv_heads=2, seq_len=4096,
                    block=64, seed=78, n_hot=8, hot_block=64, keep=0.12)
    data = gen.generate(wl)
    N, b, w, Hq = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads
    bud = dataclasses.replace(orc.default_budgets(N, b, wl.keep), diagonal_select=1)
    ses = make_session(Hq, wl.n_kv_heads, N, b, w, bud)
    Q, K, V = dev_bf16(data["Q"]), dev_bf16(data["K"]), dev_bf16(data["V"])
    O = torch.empty_like(Q)
    ses.estimate(Q, K)
    ses.build_index([IS, IS, T, IS, BC, IS, IS, BC])
    ses.prefill(Q, K, V, O)
    got = download_index(ses)
    ref, ws, _ = orc.masked_rows(data["Q"], data["K"], data["V"], b, got)
    assert np.abs(ws - 1).max() < 1e-9
    check_attention(host_f64(O), ref, "diag-blocks")
    tiles, kept = ses.prefill_counted(Q, K, V, O)
    assert kept == sum(orc.mask_count(N, b, h, got) for h in range(Hq))
    # a superset of the element-exact mask of the same offsets
    exact = make_session(Hq, wl.n_kv_heads, N, b, w, dataclasses.replace(bud, diagonal_select=0))
    exact.estimate(Q, K)
    exact.build_index([IS, IS, T, IS, BC, IS, IS, BC])
    _, kept_exact = exact.prefill_counted(Q, K, V, O)
    assert kept > kept_exact


def test_diag_blocks_whole_path_at_cfg5_128k():
    # benchmark size and launch configuration (bench.py --diagonals blocks)
    print("case diag-blocks cfg5", flush=True)
    wl = gen.WORKLOADS["cfg5"]
    data = gen.generate(wl)
    N, b, w, Hq = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads
    bud = dataclasses.replace(orc.default_budgets(N, b, wl.keep), diagonal_select=1)
    ses = make_session(Hq, wl.n_kv_heads, N, b, w, bud)
    Q, K, V = dev_bf16(data["Q"]), dev_bf16(data["K"]), dev_bf16(data["V"])
    O = torch.empty_like(Q)
    ses.estimate(Q, K)
    ses.build_index(None)
    ses.prefill(Q, K, V, O)
    v, s, blk = download_scores(ses)
    got = download_index(ses)
    print("  gpu done; patterns", got.pattern.tolist(), flush=True)
    assert_index_equal(got, orc.build_index(v, s, blk, N, b, w, bud))
    assert (got.pattern == IS).sum() >= 8 and (got.n_offs == 0).all()
    rng = np.random.Generator(np.random.Philox(key=[wl.seed, 7]))
    rows = np.unique(np.concatenate([rng.choice(N, 40, replace=False), [0, N - 1]])).astype(np.int32)
    ref, ws, _ = orc.masked_rows(data["Q"], data["K"], data["V"], b, got, rows=rows)
    assert np.abs(ws - 1).max() < 1e-9
    check_attention(host_f64(O[:, torch.from_numpy(rows.astype(np.int64)).cuda()]), ref, "diag-blocks cfg5")
