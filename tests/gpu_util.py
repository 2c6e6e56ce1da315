"""Plumbing shared by the GPU parity tests: upload bf16 bits, mirror index / score buffers."""
import numpy as np
import torch

import paper_2412_06198_amd as sa
from oracle import oracle as orc
from helpers import random_index  # noqa: F401  (used by the GPU tests through this module)

MAX_ABS, MEAN_ABS = 2e-2, 2e-3        # attention output tolerance against the fp64 oracle


def dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def host_f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def make_session(Hq, Hkv, N, b, w, bud: orc.Budgets, lazy_block_map=0):
    return sa.Session(Hq, Hkv, N, b, w, sink_blocks=bud.sink_blocks, local_blocks=bud.local_blocks,
                      k_vertical=bud.k_vertical, k_slash=bud.k_slash, k_blocks=bud.k_blocks,
                      probe_v=bud.probe_v, probe_s=bud.probe_s, lift_num=bud.lift_num,
                      lift_den=bud.lift_den, block_select=bud.block_select,
                      diagonal_select=bud.diagonal_select, lazy_block_map=lazy_block_map)


def upload_index(ses, ix: orc.Index):
    for t, a in zip(ses.index_tensors(), ix.arrays()):
        assert tuple(t.shape) == tuple(a.shape), (t.shape, a.shape)
        t.copy_(torch.from_numpy(np.ascontiguousarray(a, np.int32)))


def download_index(ses) -> orc.Index:
    torch.cuda.synchronize()
    return orc.Index(*[t.cpu().numpy() for t in ses.index_tensors()])


def upload_scores(ses, v, s, blk):
    ses.v.copy_(torch.from_numpy(np.ascontiguousarray(v, np.float32)))
    ses.s.copy_(torch.from_numpy(np.ascontiguousarray(s, np.float32)))
    ses.blk.copy_(torch.from_numpy(np.ascontiguousarray(blk, np.float32)))


def download_scores(ses):
    torch.cuda.synchronize()
    return ses.v.cpu().numpy(), ses.s.cpu().numpy(), ses.blk.cpu().numpy()


def check_attention(O_gpu, O_ref, what=""):
    d = np.abs(O_gpu - O_ref)
    assert np.isfinite(O_gpu).all(), what
    assert d.max() <= MAX_ABS, (what, float(d.max()))
    assert d.mean() <= MEAN_ABS, (what, float(d.mean()))


def assert_index_equal(a: orc.Index, b: orc.Index, heads=None):
    names = ["pattern", "n_cols", "cols", "n_offs", "offs", "rowptr", "blkcols"]
    for n, x, y in zip(names, a.arrays(), b.arrays()):
        if heads is not None:
            x, y = x[heads], y[heads]
        assert x.tobytes() == y.tobytes(), f"index array {n} differs"
