"""The decode entry point that allocates nothing (sa_sparse_decode_static) against sa_sparse_decode:
same kernels, the partial results in the library's static device array instead of the workspace.
Two calls in a row, the second on a smaller input; every call must give the bytes of the existing
entry point, which is itself checked against the fp64 oracle here and in test_gpu_decode.py."""
import numpy as np
import pytest
import torch

import paper_2412_06198_amd as sa
from harness import gen
from oracle import decode as dec
from gpu_util import dev_bf16, download_index, host_f64

pytestmark = pytest.mark.gpu


def _setup(Hq, Hkv, N, b, w, extra, keep, override, seed):
    Q, K, V = gen.random_qkv(Hq, Hkv, N + extra, 128, seed=seed)
    ses = sa.Session(Hq, Hkv, N, b, w, keep=keep, q_head_stride=(N + extra) * 128,
                     kv_head_stride=(N + extra) * 128)
    Qd, Kd, Vd = dev_bf16(Q), dev_bf16(K), dev_bf16(V)
    ses.estimate(Qd, Kd)
    ses.build_index(override)
    torch.cuda.synchronize()
    return ses, (Q, K, V), (Qd, Kd, Vd), download_index(ses)


def _both(ses, host, devs, ix, N, b, pos):
    Q, K, V = host
    Qd, Kd, Vd = devs
    q = Qd[:, pos].contiguous()
    want = torch.full_like(q, 7.0)
    ses.decode(q, Kd, Vd, pos, want)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = torch.full_like(q, -7.0)
    mid = torch.cuda.memory_allocated()
    ses.decode_static(q, Kd, Vd, pos, got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mid >= before
    assert torch.equal(got, want), f"static decode differs at pos {pos}"
    ref, _ = dec.decode_step(Q[:, pos], K, V, b, ix, N, pos)
    err = np.abs(host_f64(got) - ref)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3, (pos, float(err.max()), float(err.mean()))


def test_static_decode_two_calls_second_smaller():
    print("case static decode: 32 heads x 16 splits, then 6 heads", flush=True)
    big = _setup(32, 8, 4096, 64, 64, 8, 0.1, [h % 3 for h in range(32)], 401)
    small = _setup(6, 2, 1024, 64, 64, 5, 0.2, [h % 3 for h in range(6)], 402)
    _both(*big, 4096, 64, 4096 + 3)
    _both(*small, 1024, 64, 1024 + 2)     # fewer heads, fewer keys: stale partials of the first call lie beside it
    _both(*big, 4096, 64, 4096 + 7)
    _both(*small, 1024, 64, 1024)


def test_static_decode_needs_no_workspace():
    print("case static decode without an attached workspace", flush=True)
    ses, host, devs, ix = _setup(4, 2, 512, 64, 32, 4, 0.3, [1, 2, 0, 1], 403)
    bare = sa.sa_create(ses.cfg)              # a second context of the same shape, no workspace attached
    Qd, Kd, Vd = devs
    pos = 512 + 1
    q = Qd[:, pos].contiguous()
    want, got = torch.empty_like(q), torch.empty_like(q)
    ses.decode(q, Kd, Vd, pos, want)
    with pytest.raises(sa.SaError):
        sa.sa_sparse_decode(bare, q, Kd, Vd, ses.index(), pos, got, ses.stream())
    sa.sa_sparse_decode_static(bare, q, Kd, Vd, ses.index(), pos, got, ses.stream())
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    with pytest.raises(sa.SaError):           # the argument checks of the existing entry point apply
        sa.sa_sparse_decode_static(bare, q, Kd, Vd, ses.index(), 511, got, ses.stream())
    sa.sa_destroy(bare)
