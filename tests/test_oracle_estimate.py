"""Pins for the window estimator (Alg. 2 SumRows / SumDiagonals on the last w
query rows) and the block map (Alg. 3 blocked representation)."""
import numpy as np
import pytest
import torch

from harness import gen
from oracle import oracle as orc
from helpers import f64


def _library_window(Q, K, w, h, g):
    N = Q.shape[1]
    q, k = f64(Q)[h, N - w:], f64(K)[h // g]
    lg = (q @ k.T) / np.sqrt(128.0)
    qi = torch.arange(N - w, N)[:, None]
    lg = lg.masked_fill(torch.arange(N)[None, :] > qi, float("-inf"))
    return torch.softmax(lg, -1).numpy()


@pytest.mark.parametrize("Hq,Hkv,N,b,w", [(4, 2, 256, 32, 32), (2, 2, 320, 64, 64), (4, 1, 192, 64, 17)])
def test_estimate_against_library_softmax(Hq, Hkv, N, b, w):
    Q, K, _ = gen.random_qkv(Hq, Hkv, N, 128, seed=N + w)
    v, s, blk = orc.estimate(Q, K, b, w)
    Aw = orc.window_weights(Q, K, w)
    g = Hq // Hkv
    for h in range(Hq):
        A = _library_window(Q, K, w, h, g)
        assert np.abs(Aw[h] - A).max() <= 1e-13
        # the window rows are the last w rows of the dense weight matrix
        assert np.abs(orc.dense_weights(Q, K, h)[N - w:] - A).max() <= 1e-13
        assert np.abs(v[h] - A.sum(0)).max() <= 1e-12
        # slash score: offset o collects A[i, N-w+i-o]; that is the diagonal N-w-o of A
        want = np.array([np.trace(A, offset=N - w - o) for o in range(N)])
        assert np.abs(s[h] - want).max() <= 1e-12
    assert np.abs(v.sum(1) - w).max() <= 1e-11
    assert np.abs(s.sum(1) - w).max() <= 1e-11


def test_block_map_against_library():
    Hq, Hkv, N, b = 4, 2, 512, 64
    Q, K, _ = gen.random_qkv(Hq, Hkv, N, 128, seed=21, std=2.0)
    _, _, blk = orc.estimate(Q, K, b, 64)
    nb = N // b
    qm = f64(Q).reshape(Hq, nb, b, 128).mean(2)
    km = f64(K).reshape(Hkv, nb, b, 128).mean(2).repeat_interleave(2, 0)
    lg = torch.einsum("hrd,hcd->hrc", qm, km) / np.sqrt(128.0)
    lg = lg.masked_fill(~torch.tril(torch.ones(nb, nb, dtype=torch.bool)), float("-inf"))
    want = torch.softmax(lg, -1).numpy()
    assert np.abs(blk - want).max() <= 1e-13
    assert (blk[:, np.triu_indices(nb, 1)[0], np.triu_indices(nb, 1)[1]] == 0).all()


def test_zero_query_closed_form():
    Hq, Hkv, N, b, w = 2, 1, 256, 32, 32
    Q, K, _ = gen.random_qkv(Hq, Hkv, N, 128, seed=4)
    Q[:] = 0
    v, s, blk = orc.estimate(Q, K, b, w)
    inv = 1.0 / (np.arange(N - w, N) + 1.0)          # weight of every visible key in row i
    want_v = np.array([inv[max(0, j - (N - w)):].sum() for j in range(N)])
    assert np.abs(v[0] - want_v).max() <= 1e-14
    # offset o is seen by the rows with N-w+i-o >= 0
    want_s = np.array([inv[max(0, o - (N - w)):].sum() for o in range(N)])
    assert np.abs(s[1] - want_s).max() <= 1e-14
    nb = N // b
    for R in range(nb):
        assert np.abs(blk[0, R, :R + 1] - 1.0 / (R + 1)).max() <= 1e-15
