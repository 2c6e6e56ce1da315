"""Pins for the oracle of the decode step over the prefill index."""
import numpy as np
import torch

from harness import gen
from oracle import oracle as orc
from oracle import decode as dec
from helpers import f64

T, IS, BC = 0, 1, 2


def _setup(Hq, Hkv, N, b, w, extra, seed):
    Q, K, V = gen.random_qkv(Hq, Hkv, N + extra, 128, seed=seed)
    v, s, blk = [x.astype(np.float32) for x in orc.estimate(Q[:, :N], K[:, :N], b, w)]
    return Q, K, V, v, s, blk


def test_all_keys_index_equals_dense_row():
    # every block kept for the last row block: the decode row is the dense causal row at pos
    Hq, Hkv, N, b, w, extra = 4, 2, 256, 64, 32, 3
    nb = N // b
    Q, K, V, v, s, blk = _setup(Hq, Hkv, N, b, w, extra, 81)
    ix = orc.build_index(v, s, blk, N, b, w, orc.Budgets(1, nb, 1, 1, nb), override=[T] * Hq)
    for pos in (N, N + 2):
        q = Q[:, pos]
        o, cnt = dec.decode_step(q, K, V, b, ix, N, pos)
        qq = f64(Q[:, pos:pos + 1])
        kk = f64(K[:, :pos + 1]).repeat_interleave(Hq // Hkv, 0)
        vv = f64(V[:, :pos + 1]).repeat_interleave(Hq // Hkv, 0)
        ref = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv).numpy()[:, 0]
        assert np.abs(o - ref).max() <= 1e-12
        assert (cnt == pos + 1).all()


def test_union_counts_each_key_once_and_matches_a_boolean_mask():
    Hq, Hkv, N, b, w, extra = 6, 2, 384, 64, 32, 5
    nb = N // b
    Q, K, V, v, s, blk = _setup(Hq, Hkv, N, b, w, extra, 82)
    bud = orc.Budgets(1, 2, 40, 12, nb + 6)
    ix = orc.build_index(v, s, blk, N, b, w, bud, override=[h % 3 for h in range(Hq)])
    # hand-made overlaps on head 1 (Interval-Slash): a column inside the generated suffix is not
    # possible, but a diagonal may hit a column and offset 0 is the query itself
    pos = N + 4
    c0 = int(ix.cols[1, 0])
    ix.offs[1, 0] = 0
    ix.offs[1, 1] = pos - c0 if pos - c0 > int(ix.offs[1, 0]) else ix.offs[1, 1]
    ix.offs[1, :ix.n_offs[1]] = np.sort(ix.offs[1, :ix.n_offs[1]])
    o, cnt = dec.decode_step(Q[:, pos], K, V, b, ix, N, pos)
    for h in range(Hq):
        m = np.zeros(pos + 1, bool)
        m[N:] = True
        m[ix.cols[h, :ix.n_cols[h]]] = True
        offs = ix.offs[h, :ix.n_offs[h]]
        m[pos - offs[(offs >= 0) & (offs <= pos)]] = True
        for C in ix.blkcols[h, ix.rowptr[h, nb - 1]:ix.rowptr[h, nb]]:
            m[C * b:(C + 1) * b] = True
        assert cnt[h] == m.sum()
        qq = f64(Q[h:h + 1, pos:pos + 1])
        kk, vv = f64(K[h // 3:h // 3 + 1, :pos + 1]), f64(V[h // 3:h // 3 + 1, :pos + 1])
        ref = torch.nn.functional.scaled_dot_product_attention(
            qq, kk, vv, attn_mask=torch.from_numpy(m)[None, None, :]).numpy()[0, 0]
        assert np.abs(o[h] - ref).max() <= 1e-12


def test_zero_query_gives_the_mean_of_the_kept_values():
    Hq, Hkv, N, b, w, extra = 3, 1, 256, 64, 32, 1
    Q, K, V, v, s, blk = _setup(Hq, Hkv, N, b, w, extra, 83)
    ix = orc.build_index(v, s, blk, N, b, w, orc.Budgets(1, 1, 16, 4, 6), override=[T, IS, BC])
    q = np.zeros((Hq, 128), np.uint16)
    o, cnt = dec.decode_step(q, K, V, b, ix, N, N)
    Vf = f64(V)[0].numpy()
    for h in range(Hq):
        ks = dec.kept_keys(ix, h, N, b, N)
        assert np.abs(o[h] - Vf[ks].mean(0)).max() <= 1e-12
    # Triangular keeps the sink block and the last block of the prompt; plus the new token
    assert cnt[0] == 2 * b + 1
