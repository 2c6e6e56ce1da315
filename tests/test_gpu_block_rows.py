"""GPU parity of the per-row block rule (every row block of a Block-Cluster head keeps the same
fraction of its causal blocks): index bit-exact, attention within the usual tolerance."""
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


def _rows(bud):
    return dataclasses.replace(bud, block_select=1)


@pytest.mark.parametrize("N,b,keep", [(4096, 64, 0.10), (2048, 128, 0.3), (8192 + 128, 128, 0.07)])
def test_per_row_index_bit_exact_on_gpu_scores(N, b, keep):
    print(f"case per-row index N={N} b={b}", flush=True)
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=8, n_kv_heads=2, seq_len=N,
                    block=b, seed=N + 1, n_hot=8, hot_block=b, keep=keep)
    data = gen.generate(wl)
    bud = _rows(orc.default_budgets(N, b, keep))
    ses = make_session(8, 2, N, b, 64, bud)
    ses.estimate(dev_bf16(data["Q"]), dev_bf16(data["K"]))
    v, s, blk = download_scores(ses)
    for ov in (None, [T, IS, BC, IS, BC, T, IS, BC], [BC] * 8):
        ses.build_index(ov)
        got = download_index(ses)
        want = orc.build_index(v, s, blk, N, b, 64, bud, override=ov)
        assert_index_equal(got, want)
    nb = N // b
    assert (got.rowptr[:, nb] >= bud.k_blocks).all() and (got.rowptr[:, nb] <= bud.k_blocks + nb).all()


def test_per_row_index_ties_and_limits():
    # small-integer scores: most candidates tie at a row's boundary; budgets from one block per
    # row to every causal block
    print("case per-row ties", flush=True)
    Hq, N, b, w = 4, 1024, 64, 64
    nb = N // b
    rng = np.random.default_rng(6)
    v = rng.integers(0, 4, (Hq, N)).astype(np.float32)
    s = rng.integers(0, 3, (Hq, N)).astype(np.float32)
    blk = np.tril(rng.integers(0, 5, (Hq, nb, nb))).astype(np.float32) * 0.25
    blk[3] = 0.0                                        # every key equal (and zero)
    blk[2, 8] = np.float32(np.finfo(np.float32).max)    # a row of the largest finite key
    for kb in (nb, nb + 1, nb + 40, 77, nb * (nb + 1) // 2):
        bud = orc.Budgets(1, 2, 16, 4, kb, block_select=1)
        ses = make_session(Hq, 2, N, b, w, bud)
        upload_scores(ses, v, s, blk)
        for ov in ([BC] * Hq, [T, BC, IS, BC], None):
            ses.build_index(ov)
            assert_index_equal(download_index(ses), orc.build_index(v, s, blk, N, b, w, bud, override=ov))


@pytest.mark.parametrize("nb", [512, 1088])
def test_per_row_index_long_rows(nb):
    # rows of up to 1024 candidates (16 register slices per lane) and beyond (64 slices)
    print(f"case per-row long rows nb={nb}", flush=True)
    Hq, b, w = 2, 64, 64
    N = nb * b
    rng = np.random.default_rng(nb)
    v = rng.random((Hq, N), dtype=np.float32)
    s = rng.random((Hq, N), dtype=np.float32)
    blk = np.tril(rng.random((Hq, nb, nb), dtype=np.float32))
    blk[1] = np.round(blk[1] * 8) / 8                    # nine distinct values: long runs of ties
    bud = orc.Budgets(1, 2, 16, 4, nb * (nb + 1) // 2 // 9, block_select=1)
    ses = make_session(Hq, 1, N, b, w, bud)
    upload_scores(ses, v, s, blk)
    ses.build_index([BC] * Hq)
    assert_index_equal(download_index(ses), orc.build_index(v, s, blk, N, b, w, bud, override=[BC] * Hq))


def test_per_row_attention_matches_oracle():
    print("case per-row attention", flush=True)
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=8, n_kv_heads=2, seq_len=4096,
                    block=64, seed=77, n_hot=8, hot_block=64, keep=0.12)
    data = gen.generate(wl)
    N, b, w, Hq = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads
    bud = _rows(orc.default_budgets(N, b, wl.keep))
    ses = make_session(Hq, wl.n_kv_heads, N, b, w, bud)
    Q, K, V = dev_bf16(data["Q"]), dev_bf16(data["K"]), dev_bf16(data["V"])
    O = torch.empty_like(Q)
    ses.estimate(Q, K)
    ses.build_index([BC, BC, T, IS, BC, BC, IS, BC])
    ses.prefill(Q, K, V, O)
    got = download_index(ses)
    ref, ws, _ = orc.masked_rows(data["Q"], data["K"], data["V"], b, got)
    assert np.abs(ws - 1).max() < 1e-9
    check_attention(host_f64(O), ref, "per-row")
    tiles, kept = ses.prefill_counted(Q, K, V, O)
    assert kept == sum(orc.mask_count(N, b, h, got) for h in range(Hq))


def test_per_row_whole_path_at_cfg5_128k():
    # benchmark size and launch configuration (bench.py --block-select row): scores -> index on
    # the GPU, index bit-exact against the oracle on the same scores, attention on sampled rows
    print("case per-row cfg5", flush=True)
    wl = gen.WORKLOADS["cfg5"]
    data = gen.generate(wl)
    N, b, w, Hq = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads
    bud = _rows(orc.default_budgets(N, b, wl.keep))
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
    assert (got.pattern == BC).sum() >= 4
    rng = np.random.Generator(np.random.Philox(key=[wl.seed, 6]))
    rows = np.unique(np.concatenate([rng.choice(N, 40, replace=False), [0, N - 1]])).astype(np.int32)
    ref, ws, _ = orc.masked_rows(data["Q"], data["K"], data["V"], b, got, rows=rows)
    assert np.abs(ws - 1).max() < 1e-9
    check_attention(host_f64(O[:, torch.from_numpy(rows.astype(np.int64)).cuda()]), ref, "per-row cfg5")


@pytest.mark.parametrize("N,b,keep", [(4096, 64, 0.10), (2048, 128, 0.3)])
def test_row_normalised_key_index_bit_exact(N, b, keep):
    # block_select 2: the global top-k on blk[R][C] * (R + 1), both sides one fp32 multiplication
    print(f"case row-normalised key N={N} b={b}", flush=True)
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=8, n_kv_heads=2, seq_len=N,
                    block=b, seed=N + 5, n_hot=8, hot_block=b, keep=keep)
    data = gen.generate(wl)
    bud = dataclasses.replace(orc.default_budgets(N, b, keep), block_select=2)
    ses = make_session(8, 2, N, b, 64, bud)
    ses.estimate(dev_bf16(data["Q"]), dev_bf16(data["K"]))
    v, s, blk = download_scores(ses)
    for ov in (None, [BC] * 8):
        ses.build_index(ov)
        got = download_index(ses)
        assert_index_equal(got, orc.build_index(v, s, blk, N, b, 64, bud, override=ov))
    plain = orc.build_index(v, s, blk, N, b, 64, dataclasses.replace(bud, block_select=0), override=[BC] * 8)
    assert got.blkcols.tobytes() != plain.blkcols.tobytes()       # the key does change the choice
    # heavy ties after scaling: small integers over powers of two
    Hq, N2, b2 = 4, 1024, 64
    nb = N2 // b2
    rng = np.random.default_rng(12)
    v2 = rng.random((Hq, N2), dtype=np.float32)
    blk2 = (np.tril(rng.integers(0, 4, (Hq, nb, nb))) / 2.0 ** rng.integers(0, 3, (Hq, nb, 1))).astype(np.float32)
    for kb in (nb + 1, nb + 33, nb * (nb + 1) // 2):
        bud2 = orc.Budgets(1, 2, 16, 4, kb, block_select=2)
        ses2 = make_session(Hq, 2, N2, b2, 64, bud2)
        upload_scores(ses2, v2, v2, blk2)
        ses2.build_index([BC] * Hq)
        assert_index_equal(download_index(ses2), orc.build_index(v2, v2, blk2, N2, b2, 64, bud2, override=[BC] * Hq))
