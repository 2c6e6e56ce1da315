"""Small independent helpers for the tests (numpy / torch fp64 only)."""
import numpy as np
import torch

from harness import gen


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
