"""The three calls of the hot path recorded into one HIP graph (the estimator's side stream joins
the capture through its fork / join events) and replayed on new inputs: every replay must give the
bytes of the eager calls."""
import numpy as np
import pytest
import torch

from harness import gen
from gpu_util import dev_bf16
import paper_2412_06198_amd as sa

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("one_call,lazy", [(False, 0), (True, 0), (True, 1)])
def test_graph_replays_match_eager(one_call, lazy):
    print(f"case graph one_call={one_call} lazy={lazy}", flush=True)
    Hq, Hkv, N, b, w = 8, 2, 4096, 64, 64
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name="t", n_q_heads=Hq, n_kv_heads=Hkv, seq_len=N,
                    block=b, seed=11, n_hot=8, hot_block=b, keep=0.1)
    layers = [gen.generate(wl, seed=11 + i) for i in range(3)]
    ses = sa.Session(Hq, Hkv, N, b, w, keep=wl.keep, lazy_block_map=lazy)
    Q, K, V = (dev_bf16(layers[0][k]) for k in "QKV")
    O = torch.empty_like(Q)

    def step():
        if one_call:
            ses.estimate_and_index(Q, K, None)
        else:
            ses.estimate(Q, K)
            ses.build_index(None)
        ses.prefill(Q, K, V, O)

    def snapshot():
        torch.cuda.synchronize()
        # (lazy: the block map of a head that is not Block-Cluster keeps whatever it held)
        return [t.clone() for t in ses.index_tensors() + [ses.v, ses.s, O] + ([] if lazy else [ses.blk])]

    # eager results of every layer
    want = []
    for data in layers:
        for dst, k in ((Q, "Q"), (K, "K"), (V, "V")):
            dst.copy_(dev_bf16(data[k]))
        step()
        want.append(snapshot())
    # record once, replay on every layer (twice over), with eager work in between
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for rep in range(2):
        for data, ref in zip(layers, want):
            for dst, k in ((Q, "Q"), (K, "K"), (V, "V")):
                dst.copy_(dev_bf16(data[k]))
            for t in ses.index_tensors() + [O]:
                t.fill_(-3)                      # eager work between replays; stale outputs gone
            graph.replay()
            got = snapshot()
            for a, c in zip(got, ref):
                assert torch.equal(a, c)
