"""Small independent helpers for the tests (numpy / torch fp64 only)."""
import numpy as np
import torch

from harness import gen
from oracle import oracle as orc


def f64(bits):
    return torch.from_numpy(gen.bf16_bits_to_f32(np.ascontiguousarray(bits)).astype(np.float64))


def torch_attention(Qb, Kb, Vb, mask=None, scale=None):
    """Library fp64 attention; mask: bool [Hq,N,N] (True = keep) or None for causal."""
    q, k, v = f64(Qb), f64(Kb), f64(Vb)
    g = q.shape[0] // k.shape[0]
    k = k.repeat_interleave(g, 0)
    v = v.repeat_interleave(g, 0)
    if mask is None:
        return torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True,
                                                                scale=scale).numpy()
    m = torch.from_numpy(mask)
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=m,
                                                            scale=scale).numpy()


def numpy_mask(N, b, idx, h):
    """Boolean keep-mask of head h from an index, by one broadcast expression per part."""
    i = np.arange(N)[:, None]
    j = np.arange(N)[None, :]
    nb = N // b
    blk = np.zeros((nb, nb), bool)
    for R in range(nb):
        cs = idx.blkcols[h, idx.rowptr[h, R]:idx.rowptr[h, R + 1]]
        blk[R, cs] = True
    cols = np.zeros(N, bool)
    cols[idx.cols[h, :idx.n_cols[h]]] = True
    offs = np.zeros(N, bool)
    offs[idx.offs[h, :idx.n_offs[h]]] = True
    d = np.clip(i - j, 0, N - 1)
    return (j <= i) & (np.kron(blk, np.ones((b, b), bool)) | cols[None, :] | offs[d])


def random_index(rng, Hq, N, b, k_v, k_s, cap) -> orc.Index:
    """A hand-made index in the documented layout that no pattern produces: per head an arbitrary
    block set per row (with or without the diagonal block, possibly nothing at all, now and then a
    block above the diagonal), and arbitrary columns and offsets."""
    nb = N // b
    pattern = rng.integers(0, 3, Hq).astype(np.int32)
    n_cols = np.zeros(Hq, np.int32); cols = np.full((Hq, k_v), -1, np.int32)
    n_offs = np.zeros(Hq, np.int32); offs = np.full((Hq, k_s), -1, np.int32)
    rowptr = np.zeros((Hq, nb + 1), np.int32); blkcols = np.full((Hq, cap), -1, np.int32)
    for h in range(Hq):
        mode = rng.integers(0, 6)
        pb = [0.0, 0.05, 0.2, 0.5, 0.9, 0.3][mode]
        pdiag = [0.0, 1.0, 0.8, 0.5, 1.0, 0.0][mode]
        pos = 0
        for R in range(nb):
            cs = [C for C in range(R) if rng.random() < pb]
            if rng.random() < pdiag: cs.append(R)
            if rng.random() < 0.1 and R + 1 < nb: cs.append(int(rng.integers(R + 1, nb)))  # above the diagonal: holds no visible key
            rowptr[h, R] = pos
            blkcols[h, pos:pos + len(cs)] = cs
            pos += len(cs)
        rowptr[h, nb] = pos
        if rng.random() < 0.7:
            n = int(rng.integers(0, k_v + 1)); n_cols[h] = n
            cols[h, :n] = np.sort(rng.choice(N, n, replace=False))
        if rng.random() < 0.7:
            n = int(rng.integers(0, k_s + 1)); n_offs[h] = n
            o = np.sort(rng.choice(N, n, replace=False))
            if n and rng.random() < 0.5: o[0] = 0
            offs[h, :n] = np.unique(o)[:n] if len(np.unique(o)) == n else o
    return orc.Index(pattern, n_cols, cols, n_offs, offs, rowptr, blkcols)
