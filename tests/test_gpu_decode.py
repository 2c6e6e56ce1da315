"""GPU parity of the decode step over the prefill index against its fp64 oracle, through the C ABI.
Tolerance: the attention tolerance (max-abs 2e-2, mean-abs 2e-3 against fp64)."""
import numpy as np
import pytest
import torch

import paper_2412_06198_amd as sa
from harness import gen
from oracle import oracle as orc
from oracle import decode as dec
from gpu_util import dev_bf16, download_index, host_f64, random_index, upload_index

pytestmark = pytest.mark.gpu


def _case(Hq, Hkv, N, b, w, extra, keep, override, positions, seed, **options):
    print(f"case decode Hq={Hq} Hkv={Hkv} N={N} b={b} extra={extra} {options}", flush=True)
    Q, K, V = gen.random_qkv(Hq, Hkv, N + extra, 128, seed=seed)
    ses = sa.Session(Hq, Hkv, N, b, w, keep=keep, q_head_stride=(N + extra) * 128,
                     kv_head_stride=(N + extra) * 128, **options)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    ses.estimate(Qd, Kd)
    ses.build_index(override)
    torch.cuda.synchronize()
    ix = download_index(ses)
    for pos in positions:
        q = Qd[:, pos].contiguous()
        o = torch.full_like(q, 7.0)
        ses.decode(q, Kd, Vd, pos, o)
        torch.cuda.synchronize()
        ref, cnt = dec.decode_step(Q[:, pos], K, V, b, ix, N, pos)
        got = host_f64(o)
        err = np.abs(got - ref)
        assert err.max() <= 2e-2 and err.mean() <= 2e-3, (pos, float(err.max()), float(err.mean()))
    return ses, ix


def test_decode_patterns_and_positions():
    # every pattern, first and later decode positions, a ragged key list (not a multiple of 16 x splits)
    _case(6, 2, 1024, 64, 64, 9, 0.2, [h % 3 for h in range(6)], [1024, 1027, 1032], 301)
    _case(4, 4, 640, 128, 32, 2, 0.3, [1, 1, 2, 0], [640, 641], 302)


@pytest.mark.parametrize("options", [dict(diagonal_select=1), dict(block_select=1), dict(block_select=2),
                                     dict(block_select=1, diagonal_select=1)])
def test_decode_over_the_selection_options(options):
    # the decode step reads whatever index the prefill built: block-granular diagonals (no offset
    # list, their blocks in the last row's CSR), per-row block budgets, the row-normalised key
    _case(6, 2, 1152, 64, 64, 5, 0.2, [h % 3 for h in range(6)], [1152, 1156], 311, **options)


def test_decode_auto_patterns_planted():
    wl = gen.scaled(gen.WORKLOADS["cfg2"], seq_len=2048, n_q_heads=6, n_kv_heads=2, block=64, last_q=64,
                    n_cols=24, n_offs=12, n_hot=24, hot_block=64, window=256, seed=303)
    data = gen.generate(wl)
    N, b = wl.seq_len, wl.block
    Q, K, V = data["Q"], data["K"], data["V"]
    # the decode query is the last prompt row replayed one position later: room for one more key row
    Kx = np.concatenate([K, K[:, -1:]], axis=1)
    Vx = np.concatenate([V, V[:, -1:]], axis=1)
    ses = sa.Session(6, 2, N, b, wl.last_q, keep=0.2, kv_head_stride=(N + 1) * 128)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(Kx), dev_bf16(Vx)
    ses.estimate(Qd, Kd)
    ses.build_index(None)
    torch.cuda.synchronize()
    ix = download_index(ses)
    q = Qd[:, N - 1].contiguous()
    o = torch.empty_like(q)
    ses.decode(q, Kd, Vd, N, o)
    torch.cuda.synchronize()
    ref, cnt = dec.decode_step(Q[:, N - 1], Kx, Vx, b, ix, N, N)
    err = np.abs(host_f64(o) - ref)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3
    assert (cnt > 1).all()


def test_decode_empty_index_parts_and_argument_checks():
    Hq, Hkv, N, b, w = 2, 1, 256, 64, 32
    ses, ix = _case(Hq, Hkv, N, b, w, 1, 0.3, [1, 2], [N], 304)
    Q, K, V = gen.random_qkv(Hq, Hkv, N + 1, 128, seed=304)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    # no columns, no diagonals: only the last row block's key blocks and the new key remain
    ses.n_cols.zero_()
    ses.n_offs.zero_()
    ix2 = download_index(ses)
    q = Qd[:, N].contiguous()
    o = torch.empty_like(q)
    ses.decode(q, Kd, Vd, N, o)
    torch.cuda.synchronize()
    ref, cnt = dec.decode_step(Q[:, N], K, V, b, ix2, N, N)
    assert np.abs(host_f64(o) - ref).max() <= 2e-2
    with pytest.raises(sa.SaError):
        ses.decode(q, Kd, Vd, N - 1, o)          # a position inside the prompt is not a decode step


@pytest.mark.parametrize("seed", range(8))
def test_decode_over_hand_made_indices(seed):
    # the decode step reads the same lists as the prefill: arbitrary block sets of the last row block
    # (also none), arbitrary columns and offsets
    rng = np.random.default_rng(70000 + seed)
    b = int(rng.choice([64, 128])); nb = int(rng.integers(1, 13)); N = nb * b
    Hkv = int(rng.choice([1, 2, 3])); g = int(rng.choice([1, 2, 4])); Hq = Hkv * g
    k_v = int(rng.integers(1, min(N, 200) + 1)); k_s = int(rng.integers(1, min(N, 24) + 1))
    extra = int(rng.integers(1, 40))
    print(f"case decode hand-made index seed={seed} Hq={Hq} Hkv={Hkv} N={N} b={b} k_v={k_v} k_s={k_s} extra={extra}", flush=True)
    Q, K, V = gen.random_qkv(Hq, Hkv, N + extra, 128, seed=seed)
    ses = sa.Session(Hq, Hkv, N, b, min(64, N), sink_blocks=1, local_blocks=1, k_vertical=k_v, k_slash=k_s,
                     k_blocks=nb * (nb + 1) // 2 + nb, q_head_stride=(N + extra) * 128,
                     kv_head_stride=(N + extra) * 128)
    ix = random_index(rng, Hq, N, b, k_v, k_s, ses.cap_b)
    upload_index(ses, ix)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    for pos in sorted({N, N + extra - 1, N + int(rng.integers(0, extra))}):
        q = Qd[:, pos].contiguous()
        o = torch.full_like(q, 7.0)
        ses.decode(q, Kd, Vd, pos, o)
        torch.cuda.synchronize()
        ref, cnt = dec.decode_step(Q[:, pos], K, V, b, ix, N, pos)
        err = np.abs(host_f64(o) - ref)
        assert err.max() <= 2e-2 and err.mean() <= 2e-3, (pos, float(err.max()), float(err.mean()))
