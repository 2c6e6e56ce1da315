"""Pins for masked attention (Alg. 2 / Alg. 3 "Compute Sparse Attention")."""
import numpy as np
import pytest

from harness import gen
from oracle import oracle as orc
from helpers import numpy_mask, random_index, torch_attention

T, IS, BC = 0, 1, 2


def _scores(Q, K, b, w):
    return [x.astype(np.float32) for x in orc.estimate(Q, K, b, w)]


def test_all_keys_index_equals_dense():
    Hq, Hkv, N, b, w = 4, 2, 256, 32, 32
    nb = N // b
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=31)
    v, s, blk = _scores(Q, K, b, w)
    dense, _ = orc.dense_rows(Q, K, V)
    full = nb * (nb + 1) // 2
    cases = [
        (orc.Budgets(1, nb, 1, 1, full), [T] * Hq),          # band as wide as the sequence
        (orc.Budgets(1, 1, 1, 1, full), [BC] * Hq),          # every causal block selected
        (orc.Budgets(1, 1, 1, N, nb), [IS] * Hq),            # every diagonal offset selected
    ]
    for bud, pat in cases:
        ix = orc.build_index(v, s, blk, N, b, w, bud, override=pat)
        O, ws, kept = orc.masked_rows(Q, K, V, b, ix)
        assert np.abs(O - dense).max() <= 1e-12
        assert (kept == np.arange(1, N + 1)[None, :]).all()
        assert np.abs(ws - 1).max() <= 1e-12


@pytest.mark.parametrize("seed", [1, 2])
def test_masked_matches_library_with_numpy_mask(seed):
    Hq, Hkv, N, b, w = 6, 2, 384, 32, 32
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=seed)
    v, s, blk = _scores(Q, K, b, w)
    bud = orc.Budgets(1, 2, 9, 5, 30)
    ix = orc.build_index(v, s, blk, N, b, w, bud, override=[T, IS, BC, IS, BC, T])
    O, ws, kept = orc.masked_rows(Q, K, V, b, ix)
    mask = np.stack([numpy_mask(N, b, ix, h) for h in range(Hq)])
    ref = torch_attention(Q, K, V, mask=mask)
    assert np.abs(O - ref).max() <= 1e-12
    assert np.abs(ws - 1).max() <= 1e-12          # every row keeps at least its diagonal block
    assert (kept == mask.sum(2)).all()
    for h in range(Hq):
        assert orc.mask_count(N, b, h, ix) == mask[h].sum()
    rows = np.array([0, 31, 32, 200, 383], np.int32)
    Or, _, _ = orc.masked_rows(Q, K, V, b, ix, rows=rows)
    assert np.abs(Or - ref[:, rows]).max() <= 1e-12


def test_union_counts_a_key_once():
    # a column that already lies in a kept block, an offset that duplicates a column hit
    Hq, Hkv, N, b = 1, 1, 128, 32
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=8)
    nb = N // b

    def idx(cols, offs):
        kv, ks = max(len(cols), 1), max(len(offs), 1)
        c = np.full((1, kv), -1, np.int32); c[0, :len(cols)] = cols
        o = np.full((1, ks), -1, np.int32); o[0, :len(offs)] = offs
        return orc.Index(np.array([IS], np.int32), np.array([len(cols)], np.int32), c,
                         np.array([len(offs)], np.int32), o,
                         np.arange(nb + 1, dtype=np.int32)[None].copy(),
                         np.arange(nb, dtype=np.int32)[None].copy())

    base, _, kb = orc.masked_rows(Q, K, V, b, idx([5], [40]))
    # offset 0 lies inside the always-kept diagonal block: adding it changes nothing
    plus, _, kp = orc.masked_rows(Q, K, V, b, idx([5], [0, 40]))
    assert (kb == kp).all() and np.abs(base - plus).max() == 0
    # row 10: column 5 is inside the diagonal block of row block 0 -> 11 keys, not 12
    assert kb[0, 10] == 11
    # row 45: keys 32..45 of the block, column 5, and offset 40 -> key 5 again: counted once
    assert kb[0, 45] == 14 + 1
    # row 50: keys 32..50, column 5, offset 40 -> key 10
    assert kb[0, 50] == 19 + 1 + 1
    mask = numpy_mask(N, b, idx([5], [40]), 0)[None]
    assert np.abs(base - torch_attention(Q, K, V, mask=mask)).max() <= 1e-12


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_hand_made_indices_and_rows_that_keep_nothing(seed):
    # indices no pattern produces (rows without their diagonal block, empty rows and heads, blocks
    # above the diagonal): the oracle against library attention under an independently built mask;
    # a row that keeps no key is a row of zeros with weight sum 0
    rng = np.random.default_rng(90000 + seed)
    Hq, Hkv, N, b = 4, 2, 256, 32
    nb = N // b
    Q, K, V = gen.random_qkv(Hq, Hkv, N, 128, seed=seed)
    ix = random_index(rng, Hq, N, b, 20, 6, nb * (nb + 1) // 2 + nb)
    O, ws, kept = orc.masked_rows(Q, K, V, b, ix)
    mask = np.stack([numpy_mask(N, b, ix, h) for h in range(Hq)])
    assert (kept == mask.sum(2)).all()
    empty = kept == 0
    assert empty.any() and (~empty).any()
    safe = mask.copy()
    safe[empty, 0] = True                     # the library has no convention for an empty row
    ref = torch_attention(Q, K, V, mask=safe)
    assert np.abs(O[~empty] - ref[~empty]).max() <= 1e-12
    assert np.abs(ws[~empty] - 1).max() <= 1e-12
    assert (O[empty] == 0).all() and (ws[empty] == 0).all()
    for h in range(Hq):
        assert orc.mask_count(N, b, h, ix) == mask[h].sum()
