"""fp64 oracle of the offline pattern search (Kernel-Aware Sparse Pattern Search Algorithm, Alg. 1).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

Per head the candidates are the three patterns; the search space of a candidate is one integer
size x (the paper leaves the parametrisation open):
    Triangular       local_blocks = x,              1 <= x <= nb
    Interval-Slash   k_slash = x, k_vertical = min(N, 32 x),   1 <= x <= max(1, N/32)
    Block-Cluster    k_blocks = x,                  nb <= x <= nb (nb+1) / 2
FLOPs(S_i) = 4 d |M|, |M| = kept (query, key) pairs of the index built from S_i, so the target and
its tolerance are given in pairs.  RefineSearchSpace is a bisection on x (|M| is monotone in x).
Evaluate Patterns: the dense causal output of the head against the sparse output of every refined
candidate, Frobenius norm of the difference, the smallest wins (ties: lowest pattern id).
"""
from __future__ import annotations

import numpy as np

from . import oracle as orc

PATTERNS = (orc.TRIANGULAR, orc.INTERVAL_SLASH, orc.BLOCK_CLUSTER)


def candidate_range(pattern: int, N: int, b: int):
    nb = N // b
    if pattern == orc.TRIANGULAR:
        return 1, nb
    if pattern == orc.INTERVAL_SLASH:
        return 1, max(1, N // 32)
    return nb, nb * (nb + 1) // 2


def candidate_budgets(pattern: int, x: int, N: int, b: int, sink_blocks: int) -> orc.Budgets:
    nb = N // b
    if pattern == orc.TRIANGULAR:
        return orc.Budgets(sink_blocks, x, 1, 1, nb)
    if pattern == orc.INTERVAL_SLASH:
        return orc.Budgets(sink_blocks, 1, min(N, 32 * x), x, nb)
    return orc.Budgets(sink_blocks, 1, 1, 1, x)


def refine(pairs_of, lo: int, hi: int, target: int, eps: int):
    """Bisection on the size x in [lo, hi] of a candidate whose pair count pairs_of(x) does not
    decrease with x.  Returns (x, pairs): the first probe within eps of the target, else of the two
    sizes that bracket the target the one closer to it (the smaller on a tie)."""
    p_lo = pairs_of(lo)
    if p_lo >= target or abs(p_lo - target) <= eps or lo == hi:
        return lo, p_lo
    p_hi = pairs_of(hi)
    if p_hi <= target or abs(p_hi - target) <= eps:
        return hi, p_hi
    while hi - lo > 1:
        mid = (lo + hi) // 2
        p = pairs_of(mid)
        if abs(p - target) <= eps:
            return mid, p
        if p < target:
            lo, p_lo = mid, p
        else:
            hi, p_hi = mid, p
    return (lo, p_lo) if target - p_lo <= p_hi - target else (hi, p_hi)


def search_patterns(Q, K, V, v, s, blk, b: int, w: int, sink_blocks: int, target_pairs: int,
                    eps_pairs: int, scale=None):
    """Alg. 1 for every head.  Q [Hq,N,d], K, V [Hkv,N,d] bf16 bit patterns; v, s [Hq,N] and blk
    [Hq,nb,nb] the estimator's scores.  Returns one dict per head: pattern, param[3], pairs[3],
    err[3] (candidates in pattern-id order)."""
    Hq, N, d = Q.shape
    g = Hq // K.shape[0]
    out = []
    for h in range(Hq):
        Qh, Kh, Vh = Q[h:h + 1], K[h // g:h // g + 1], V[h // g:h // g + 1]
        vh, sh, bh = v[h:h + 1], s[h:h + 1], blk[h:h + 1]
        dense, _ = orc.dense_rows(Qh, Kh, Vh, scale=scale)
        res = {"param": [], "pairs": [], "err": []}
        for p in PATTERNS:
            def sparse(x, p=p):
                bud = candidate_budgets(p, x, N, b, sink_blocks)
                idx = orc.build_index(vh, sh, bh, N, b, w, bud, override=[p])
                return orc.masked_rows(Qh, Kh, Vh, b, idx, scale=scale)

            lo, hi = candidate_range(p, N, b)
            x, pairs = refine(lambda x: int(sparse(x)[2].sum()), lo, hi, target_pairs, eps_pairs)
            O = sparse(x)[0]
            res["param"].append(x)
            res["pairs"].append(pairs)
            res["err"].append(float(np.sqrt(((O - dense) ** 2).sum())))
        res["pattern"] = int(np.argmin(res["err"]))  # first minimum: ties go to the lowest id
        out.append(res)
    return out
