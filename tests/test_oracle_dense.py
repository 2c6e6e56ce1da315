"""Pins for the dense oracle (Alg. 1 A_dense with the causal mask of Alg. 2)."""
import numpy as np
import pytest
import torch

from harness import gen
from oracle import oracle as orc
from helpers import f64, torch_attention


@pytest.mark.parametrize("Hq,Hkv,N", [(2, 2, 33), (4, 2, 200), (4, 1, 129)])
def test_dense_matches_library_fp64(Hq, Hkv, N):
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=N)
    O, ws = orc.dense_rows(Q, K, V)
    ref = torch_attention(Q, K, V)
    assert np.abs(O - ref).max() <= 1e-12
    assert np.abs(ws - 1.0).max() <= 1e-12


def test_dense_row_subset_and_scale():
    Q, K, V = gen.random_qkv(4, 2, 150, 128, seed=5)
    rows = np.array([0, 1, 77, 149], np.int32)
    O, ws = orc.dense_rows(Q, K, V, scale=0.31, rows=rows)
    ref = torch_attention(Q, K, V, scale=0.31)[:, rows]
    assert np.abs(O - ref).max() <= 1e-12


def test_dense_zero_query_is_prefix_mean():
    Q, K, V = gen.random_qkv(2, 1, 96, 128, seed=9)
    Q[:] = 0
    O, _ = orc.dense_rows(Q, K, V)
    v = f64(V).numpy()[0]
    want = np.cumsum(v, 0) / np.arange(1, 97)[:, None]
    assert np.abs(O[0] - want).max() <= 1e-12
    assert np.abs(O[1] - want).max() <= 1e-12


def test_dense_one_hot_keys_pick_argmax():
    # K[j] = e_j, Q[i] = big * e_{t(i)}, t(i) <= i: weights collapse on key t(i)
    N, d = 100, 128
    Kf = np.zeros((1, N, d), np.float32)
    Kf[0, np.arange(N), np.arange(N) % d] = 1.0
    Kf[0, np.arange(N), (np.arange(N) // d) + 64] += 0.0
    rng = np.random.default_rng(0)
    t = np.array([rng.integers(max(0, i - 60), i + 1) for i in range(N)])
    Qf = np.zeros((1, N, d), np.float32)
    Qf[0, np.arange(N), t % d] = 4096.0
    Vb = gen.random_qkv(1, 1, N, d, seed=3)[2]
    O, _ = orc.dense_rows(gen.f32_to_bf16_bits(Qf), gen.f32_to_bf16_bits(Kf), Vb)
    want = f64(Vb).numpy()[0][t]
    assert np.abs(O[0] - want).max() <= 1e-12


def test_dense_weights_rows_sum_to_one_and_match_library():
    Q, K, V = gen.random_qkv(2, 1, 64, 128, seed=11)
    A = orc.dense_weights(Q, K, 1)
    assert np.abs(A.sum(1) - 1).max() <= 1e-12
    q, k = f64(Q)[1], f64(K)[0]
    lg = (q @ k.T) / np.sqrt(128.0)
    lg = lg.masked_fill(~torch.tril(torch.ones(64, 64, dtype=torch.bool)), float("-inf"))
    assert np.abs(A - torch.softmax(lg, -1).numpy()).max() <= 1e-13
