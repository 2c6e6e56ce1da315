"""GPU parity on the edges of the boundary: strides, custom scale, a non-default stream, the
smallest shapes, empty index parts, and the last-query window at its limits."""
import numpy as np
import pytest
import torch

import paper_2412_06198_amd as sa
from harness import gen
from oracle import oracle as orc
from gpu_util import (assert_index_equal, check_attention, dev_bf16, download_index, download_scores,
                      host_f64, make_session, upload_index)

pytestmark = pytest.mark.gpu


def _check_scores(got, ref, w):
    for name, g, r in zip("v s blk".split(), got, ref):
        tol = 1e-3 * np.abs(r) + 1e-6 * w
        bad = np.abs(g.astype(np.float64) - r) > tol
        assert not bad.any(), (name, int(bad.sum()), float(np.abs(g - r).max()))


def _run_all(ses, Qd, Kd, Vd, Od, override):
    ses.estimate(Qd, Kd)
    ses.build_index(override)
    ses.prefill(Qd, Kd, Vd, Od)
    torch.cuda.synchronize()


def test_strided_layout_and_custom_scale():
    # Q/K/V/O rows padded to 160 elements and heads padded by 3 rows: strides come from the config
    print("case strides", flush=True)
    Hq, Hkv, N, b, w, d, rs = 4, 2, 512, 64, 64, 128, 160
    scale = 0.07
    Q, K, V = gen.random_qkv(Hq, Hkv, N, d, seed=11)
    bud = orc.default_budgets(N, b, 0.3)
    ses = sa.Session(Hq, Hkv, N, b, w, sink_blocks=bud.sink_blocks, local_blocks=bud.local_blocks,
                     k_vertical=bud.k_vertical, k_slash=bud.k_slash, k_blocks=bud.k_blocks,
                     softmax_scale=scale, q_row_stride=rs, q_head_stride=(N + 3) * rs,
                     kv_row_stride=rs, kv_head_stride=(N + 3) * rs)

    def padded(bits, H):
        t = torch.zeros((H, N + 3, rs), dtype=torch.bfloat16, device="cuda")
        t[:, :N, :d] = dev_bf16(bits)
        return t

    Qd, Kd, Vd = padded(Q, Hq), padded(K, Hkv), padded(V, Hkv)
    Od = torch.full_like(Qd, 7.0)
    ov = [0, 1, 2, 1]
    _run_all(ses, Qd, Kd, Vd, Od, ov)
    _check_scores(download_scores(ses), orc.estimate(Q, K, b, w, scale=scale), w)
    ix = download_index(ses)
    v, s, blk = download_scores(ses)
    assert_index_equal(ix, orc.build_index(v, s, blk, N, b, w, bud, override=ov))
    ref, _, _ = orc.masked_rows(Q, K, V, b, ix, scale=scale)
    check_attention(host_f64(Od[:, :N, :d]), ref, "strided")
    # nothing outside the [N][d] window of O is written
    assert (Od[:, N:, :] == 7.0).all() and (Od[:, :, d:] == 7.0).all()


def test_non_default_stream():
    print("case stream", flush=True)
    Hq, Hkv, N, b, w = 4, 2, 1024, 128, 64
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=12)
    bud = orc.default_budgets(N, b, 0.4)
    ses = make_session(Hq, Hkv, N, b, w, bud)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    Od = torch.empty_like(Qd)
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for _ in range(3):                     # back-to-back calls on one stream reuse the workspace in order
            ses.estimate(Qd, Kd)
            ses.build_index(None)
            ses.prefill(Qd, Kd, Vd, Od)
    st.synchronize()
    _check_scores(download_scores(ses), orc.estimate(Q, K, b, w), w)
    ix = download_index(ses)
    v, s, blk = download_scores(ses)
    assert_index_equal(ix, orc.build_index(v, s, blk, N, b, w, bud))
    ref, _, _ = orc.masked_rows(Q, K, V, b, ix)
    check_attention(host_f64(Od), ref, "stream")


@pytest.mark.parametrize("Hq,Hkv,N,b,w", [(1, 1, 64, 64, 1), (2, 1, 128, 128, 64), (3, 3, 128, 64, 5),
                                          (8, 1, 192, 64, 64)])
def test_smallest_shapes(Hq, Hkv, N, b, w):
    print(f"case tiny Hq={Hq} Hkv={Hkv} N={N} b={b} w={w}", flush=True)
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=N + w + Hq)
    nb = N // b
    bud = orc.Budgets(1, 1, min(7, N), min(3, N), nb + 1 if nb > 1 else nb)
    ses = make_session(Hq, Hkv, N, b, w, bud)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    Od = torch.empty_like(Qd)
    for ov in ([h % 3 for h in range(Hq)], [(h + 1) % 3 for h in range(Hq)], None):
        _run_all(ses, Qd, Kd, Vd, Od, ov)
        _check_scores(download_scores(ses), orc.estimate(Q, K, b, w), w)
        ix = download_index(ses)
        v, s, blk = download_scores(ses)
        assert_index_equal(ix, orc.build_index(v, s, blk, N, b, w, bud, override=ov))
        ref, _, _ = orc.masked_rows(Q, K, V, b, ix)
        check_attention(host_f64(Od), ref, f"tiny {ov}")


def test_empty_index_parts():
    # an index with no columns, no offsets and only the diagonal blocks: every row still attends itself
    print("case empty parts", flush=True)
    Hq, Hkv, N, b, w = 2, 1, 512, 64, 64
    nb = N // b
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=13)
    bud = orc.Budgets(0, 1, 4, 2, nb)
    ses = make_session(Hq, Hkv, N, b, w, bud)
    cap = ses.cap_b
    rowptr = np.tile(np.arange(nb + 1, dtype=np.int32), (Hq, 1))
    blkcols = np.full((Hq, cap), -1, np.int32)
    blkcols[:, :nb] = np.arange(nb, dtype=np.int32)
    ix = orc.Index(np.full(Hq, 1, np.int32), np.zeros(Hq, np.int32), np.full((Hq, 4), -1, np.int32),
                   np.zeros(Hq, np.int32), np.full((Hq, 2), -1, np.int32), rowptr, blkcols)
    upload_index(ses, ix)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    Od = torch.empty_like(Qd)
    ses.prefill(Qd, Kd, Vd, Od)
    torch.cuda.synchronize()
    ref, _, _ = orc.masked_rows(Q, K, V, b, ix)
    check_attention(host_f64(Od), ref, "diagonal blocks only")


@pytest.mark.parametrize("Hq,Hkv,N,b", [(3, 3, 704, 64), (10, 5, 640, 128), (6, 1, 576, 64),
                                        (16, 16, 384, 128), (12, 6, 1088, 64), (64, 8, 512, 64),
                                        (40, 5, 384, 128), (128, 16, 256, 64), (9, 9, 448, 64)])
def test_head_counts_off_the_queue_grid(Hq, Hkv, N, b):
    # KV head counts that do not divide the eight work queues (and row-block counts that do not
    # divide the queues of a KV head): every (head, row block) must still be computed exactly once
    print(f"case heads Hq={Hq} Hkv={Hkv} N={N} b={b}", flush=True)
    w = 64
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=100 + Hq)
    bud = orc.default_budgets(N, b, 0.3)
    ses = make_session(Hq, Hkv, N, b, w, bud)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    Od = torch.full_like(Qd, 7.0)
    ov = [h % 3 for h in range(Hq)]
    _run_all(ses, Qd, Kd, Vd, Od, ov)
    ix = download_index(ses)
    v, s, blk = download_scores(ses)
    assert_index_equal(ix, orc.build_index(v, s, blk, N, b, w, bud, override=ov))
    ref, _, _ = orc.masked_rows(Q, K, V, b, ix)
    check_attention(host_f64(Od), ref, f"heads {Hq}/{Hkv}")


def test_rows_with_a_handful_of_keys_and_large_values():
    # Rows that keep one to four keys, with V entries of magnitude 3.5 .. 4.4 planted in 6 % of V:
    # the output is a convex combination of a few V rows, so the bf16 rounding of the dominant
    # weight (2^-9 relative) shows at full size, 4.4 * 2^-9 = 0.009, on top of the output's own
    # rounding (2^-6 at |O| in [4, 8)) unless the weights are normalised by the sum of what the
    # matrix pipe actually multiplies.  Heads served by the diagonal phase only, by gather tiles
    # only, and by both; no blocks at all.
    print("case few-key rows", flush=True)
    Hq, Hkv, N, b, w = 4, 2, 512, 128, 64
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=2651)
    rng = np.random.default_rng(77)
    Vf = gen.bf16_bits_to_f32(V)
    big = rng.random(Vf.shape) < 0.06
    Vf[big] = (rng.uniform(3.5, 4.4, Vf.shape) * rng.choice([-1.0, 1.0], Vf.shape))[big].astype(np.float32)
    V = gen.f32_to_bf16_bits(Vf)
    k_v, k_s, nb = 4, 4, N // b
    bud = orc.Budgets(1, 1, k_v, k_s, nb * (nb + 1) // 2 + nb)
    ses = make_session(Hq, Hkv, N, b, w, bud)
    cols = np.full((Hq, k_v), -1, np.int32)
    offs = np.full((Hq, k_s), -1, np.int32)
    want_offs = [[14, 233, 288, 505], [], [0, 1], [0, 130, 257]]
    want_cols = [[], [3, 200, 410], [0], [5, 300]]
    for h in range(Hq):
        offs[h, :len(want_offs[h])] = want_offs[h]
        cols[h, :len(want_cols[h])] = want_cols[h]
    ix = orc.Index(np.array([1, 0, 1, 1], np.int32),
                   np.array([len(c) for c in want_cols], np.int32), cols,
                   np.array([len(o) for o in want_offs], np.int32), offs,
                   np.zeros((Hq, nb + 1), np.int32), np.full((Hq, ses.cap_b), -1, np.int32))
    upload_index(ses, ix)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    Od = torch.full_like(Qd, 7.0)
    ses.prefill(Qd, Kd, Vd, Od)
    torch.cuda.synchronize()
    ref, _, kept = orc.masked_rows(Q, K, V, b, ix)
    assert int(kept.max()) <= 5 and int((kept == 0).sum()) > 0  # a handful of keys; some rows keep none
    assert float(np.abs(ref).max()) > 4.0                       # and the case does reach the large outputs
    check_attention(host_f64(Od), ref, "few-key rows")
