"""fp64 oracle of one decode step over the prefill index (the paper's "improvements in the decoding
phase" are a single clause of its abstract and introduction; the problem statement only fixes the
query shape [B, 1, H]).  TEST INFRASTRUCTURE ONLY, like the rest of this package.

Reading: the prompt of N tokens was prefilled with index I.  The query at position pos >= N (the
(pos+1)-th token; K and V hold rows 0..pos) attends, per query head, the union of
  * every generated key N..pos (itself included),
  * the selected key columns of I,
  * the keys pos - o for the selected diagonal offsets o of I,
  * the keys of the key blocks that I keeps for the last row block of the prompt,
each key once, with the same scaled softmax as the prefill.
"""
from __future__ import annotations

import numpy as np

from . import oracle as orc


def _f64(bits):
    return (np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def kept_keys(idx: orc.Index, h: int, N: int, b: int, pos: int) -> np.ndarray:
    """Sorted key positions the decode query of head h attends."""
    nb = N // b
    keys = set(range(N, pos + 1))
    keys.update(int(c) for c in idx.cols[h, :max(int(idx.n_cols[h]), 0)] if 0 <= c < N)
    for o in idx.offs[h, :max(int(idx.n_offs[h]), 0)]:
        if o >= 0 and 0 <= pos - int(o) <= pos:
            keys.add(pos - int(o))
    for C in idx.blkcols[h, idx.rowptr[h, nb - 1]:idx.rowptr[h, nb]]:
        if C >= 0:
            keys.update(range(int(C) * b, int(C) * b + b))
    return np.array(sorted(keys), dtype=np.int64)


def decode_step(q, K, V, b: int, idx: orc.Index, N: int, pos: int, scale=None):
    """q [Hq,d], K, V [Hkv,>=pos+1,d] bf16 bit patterns.  Returns (o [Hq,d] fp64, kept counts [Hq])."""
    Hq, d = q.shape
    g = Hq // K.shape[0]
    scale = orc.default_scale(d) if scale is None else scale
    qf, Kf, Vf = _f64(q), _f64(K), _f64(V)
    out = np.empty((Hq, d), np.float64)
    cnt = np.empty(Hq, np.int64)
    for h in range(Hq):
        ks = kept_keys(idx, h, N, b, pos)
        s = scale * (Kf[h // g, ks] @ qf[h])
        p = np.exp(s - s.max())
        out[h] = (p / p.sum()) @ Vf[h // g, ks]
        cnt[h] = ks.size
    return out, cnt
