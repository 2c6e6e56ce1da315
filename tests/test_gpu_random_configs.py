"""Whole path on seeded random small configurations: shapes, GQA ratios, budgets, window sizes,
pattern overrides and both selection options drawn together, so that their combinations are
exercised (scores by tolerance, index bit-exact on the GPU's scores, attention on all rows, kept
pairs counted)."""
import numpy as np
import pytest
import torch

from harness import gen
from oracle import oracle as orc
from gpu_util import (assert_index_equal, check_attention, dev_bf16, download_index,
                      download_scores, host_f64, make_session)

pytestmark = pytest.mark.gpu


def _draw(rng):
    b = int(rng.choice([64, 128]))
    nb = int(rng.integers(1, 25))
    N = nb * b
    Hkv = int(rng.choice([1, 2, 3, 4]))
    g = int(rng.choice([1, 2, 4]))
    w = int(rng.integers(1, 65))
    w = min(w, N)
    all_blocks = nb * (nb + 1) // 2
    bud = orc.Budgets(
        sink_blocks=int(rng.integers(0, 3)), local_blocks=int(rng.integers(1, nb + 1)),
        k_vertical=int(rng.integers(1, min(N, 300) + 1)), k_slash=int(rng.integers(1, min(N, 40) + 1)),
        k_blocks=int(rng.integers(nb, all_blocks + 1)), probe_v=int(rng.integers(1, 7)),
        probe_s=int(rng.integers(1, 7)), lift_num=int(rng.integers(1, 6)), lift_den=int(rng.integers(1, 3)),
        block_select=int(rng.integers(0, 3)), diagonal_select=int(rng.integers(0, 2)))
    Hq = Hkv * g
    ov = None if rng.random() < 0.4 else [int(x) for x in rng.integers(-1, 3, Hq)]
    return Hq, Hkv, N, b, w, bud, ov


@pytest.mark.parametrize("seed", range(64))
def test_random_configuration(seed):
    rng = np.random.default_rng(1000 + seed)
    Hq, Hkv, N, b, w, bud, ov = _draw(rng)
    print(f"case random seed={seed} Hq={Hq} Hkv={Hkv} N={N} b={b} w={w} {bud} ov={ov}", flush=True)
    Qp, Kp, Vp = gen.random_qkv(Hq, Hkv, N, 128, seed=seed)
    ses = make_session(Hq, Hkv, N, b, w, bud)
    Qd, Kd, Vd = dev_bf16(Qp), dev_bf16(Kp), dev_bf16(Vp)
    O = torch.empty_like(Qd)
    if seed % 2:
        ses.estimate_and_index(Qd, Kd, ov)
    else:
        ses.estimate(Qd, Kd)
        ses.build_index(ov)
    ses.prefill(Qd, Kd, Vd, O)
    v, s, blk = download_scores(ses)
    for nm, g_, r_ in zip("v s blk".split(), (v, s, blk), orc.estimate(Qp, Kp, b, w)):
        bad = np.abs(g_ - r_) > 1e-3 * np.abs(r_) + 1e-6 * w
        assert not bad.any(), (nm, int(bad.sum()))
    got = download_index(ses)
    assert_index_equal(got, orc.build_index(v, s, blk, N, b, w, bud, override=ov))
    ref, ws, _ = orc.masked_rows(Qp, Kp, Vp, b, got)
    assert np.abs(ws - 1).max() < 1e-9
    check_attention(host_f64(O), ref, f"random {seed}")
    tiles, kept = ses.prefill_counted(Qd, Kd, Vd, O)
    assert kept == sum(orc.mask_count(N, b, h, got) for h in range(Hq))
    # the one-call form that computes the block map for the Block-Cluster heads only: same index
    lz = make_session(Hq, Hkv, N, b, w, bud, lazy_block_map=1)
    lz.estimate_and_index(Qd, Kd, ov)
    assert_index_equal(download_index(lz), got)
