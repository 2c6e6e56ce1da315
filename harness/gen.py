"""Seeded synthetic Q/K/V with planted attention structure.

The paper evaluates on Llama-3.1-8B-Instruct prompts (Experimental Results,
"Model"); neither weights nor prompts are available, so these inputs stand in:
the layer shape of that model (32 query / 8 KV heads, head_dim 128) and, per
head, one of the three structures the paper names in its contributions list
(Triangular, Interval-Slash, Block-Cluster).

Everything is host numpy: Philox-seeded fp32 draws, rounded to bf16
(round-to-nearest-even) at the end.  The same uint16 bit arrays are handed to
the CPU oracle and uploaded to the GPU.  Nothing here evaluates attention.

Planting (the API has no bias input, so a "+beta logit bias" is realised in Q
and K themselves, beta = 3, a = c = sqrt(beta*sqrt(d))):
  * base Q0, K0, V ~ N(0,1); dims [96,128) of Q0 and K0 are zeroed and
    reserved for the plants (V is untouched);
  * column plant (sink keys, vertical columns): one reserved channel per query
    head of the KV group, dim 96 + (h mod 4): K[j,ch] = a on planted keys,
    Q_h[i,ch] = c on every query row;
  * diagonal plant (slash offset o): Q_h[i] += (beta*sqrt(d)/96) * K0[i-o];
  * block plant: a random unit code u in dims [100,128); K[j] += a*u on the
    keys of the block, Q_h[i] += c*u on the query rows that should see it.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

BETA = 3.0
PLANT_LO = 96          # first reserved dim
CODE_LO = 100          # first dim of block codes

TRIANGULAR, INTERVAL_SLASH, BLOCK_CLUSTER, UNPLANTED = 0, 1, 2, -1


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class HeadPlant:
    pattern: int = UNPLANTED
    sinks: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    cols: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    offs: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    hot: np.ndarray = field(default_factory=lambda: np.zeros((0, 2), np.int64))
    hot_block: int = 0
    window: int = 0


@dataclass
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    seq_len: int
    head_dim: int
    block: int
    last_q: int
    keep: float
    seed: int
    # planted structure
    mix: str = "none"            # "cfg1" | "mod3" | "tiib" | "none"
    n_cols: int = 16
    n_offs: int = 8
    n_hot: int = 32
    hot_block: int = 64
    hot_bands: int = 0           # 0: hot blocks anywhere; >0: clustered on that many query bands
    window: int = 1024
    n_sinks: int = 4


# The five configurations of the benchmark definition.  keep/block/last_q where
# the definition leaves them open: cfg2 keep = 2*1024/N (the planted band),
# cfg2/cfg3 block 64, cfg4 Block-Cluster heads 32 hot 128x128 blocks.
WORKLOADS = {
    "cfg1": Workload("cfg1", 4, 4, 4096, 128, 64, 64, 0.10, 0, mix="cfg1"),
    "cfg2": Workload("cfg2", 32, 8, 16384, 128, 64, 64, 0.125, 2000, mix="mod3"),
    "cfg3": Workload("cfg3", 32, 8, 32768, 128, 64, 64, 0.06, 3000, mix="tiib"),
    "cfg4": Workload("cfg4", 32, 8, 65536, 128, 128, 64, 0.04, 4000, mix="tiib",
                     n_cols=32, n_offs=16, n_hot=32, hot_block=128),
    "cfg5": Workload("cfg5", 32, 8, 131072, 128, 128, 64, 0.03, 5000, mix="tiib",
                     n_cols=32, n_offs=16, n_hot=128, hot_block=128, hot_bands=4),
}


def scaled(base: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (used for small test sizes)."""
    d = dict(base.__dict__)
    d.update(kw)
    return Workload(**d)


def _assign_patterns(wl: Workload) -> list[int]:
    g = wl.n_q_heads // wl.n_kv_heads
    out = []
    for h in range(wl.n_q_heads):
        if wl.mix == "cfg1":
            out.append(INTERVAL_SLASH)
        elif wl.mix == "mod3":
            out.append(h % 3)
        elif wl.mix == "tiib":
            out.append([TRIANGULAR, INTERVAL_SLASH, INTERVAL_SLASH, BLOCK_CLUSTER][h % 4])
        else:
            out.append(UNPLANTED)
    return out


def draw_plants(wl: Workload, seed: int | None = None) -> list[HeadPlant]:
    """Draw the planted structure of every head (no tensor data)."""
    seed = wl.seed if seed is None else seed
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x9E3779B9]))
    N, w = wl.seq_len, wl.last_q
    plants = []
    for h, pat in enumerate(_assign_patterns(wl)):
        p = HeadPlant(pattern=pat)
        if wl.mix == "cfg1":
            p.sinks = np.arange(wl.n_sinks, dtype=np.int64)
            p.offs = np.array([0, 64, 512], dtype=np.int64)
        elif pat == TRIANGULAR:
            p.sinks = np.arange(wl.n_sinks, dtype=np.int64)
            p.window = min(wl.window, N)
        elif pat == INTERVAL_SLASH:
            # columns and offsets are drawn where every window row sees them
            p.cols = np.sort(rng.choice(N - w, size=wl.n_cols, replace=False)).astype(np.int64)
            p.offs = np.sort(rng.choice(N - w + 1, size=wl.n_offs, replace=False)).astype(np.int64)
        elif pat == BLOCK_CLUSTER:
            hb = wl.hot_block
            nhb = N // hb
            if wl.hot_bands > 0:
                bands = rng.choice(np.arange(1, nhb), size=wl.hot_bands, replace=False)
                per = wl.n_hot // wl.hot_bands
                hot = []
                for R in np.sort(bands):
                    k = min(per, int(R))
                    cs = rng.choice(int(R), size=k, replace=False)
                    hot += [(int(R), int(c)) for c in np.sort(cs)]
                p.hot = np.array(hot, dtype=np.int64).reshape(-1, 2)
            else:
                # uniform over strictly-below-diagonal blocks
                total = nhb * (nhb - 1) // 2
                k = min(wl.n_hot, total)
                flat = np.sort(rng.choice(total, size=k, replace=False))
                R = np.floor((1 + np.sqrt(1 + 8 * flat.astype(np.float64))) / 2).astype(np.int64)
                R = np.where(R * (R - 1) // 2 > flat, R - 1, R)
                R = np.where((R + 1) * R // 2 <= flat, R + 1, R)
                C = flat - R * (R - 1) // 2
                p.hot = np.stack([R, C], axis=1).astype(np.int64)
            p.hot_block = hb
        plants.append(p)
    return plants


def generate(wl: Workload, seed: int | None = None, plants: list[HeadPlant] | None = None):
    """Return dict(Q,K,V) of uint16 bf16 bit patterns plus the planted structure.

    Shapes: Q [Hq,N,d], K and V [Hkv,N,d], C-contiguous.
    """
    seed = wl.seed if seed is None else seed
    Hq, Hkv, N, d = wl.n_q_heads, wl.n_kv_heads, wl.seq_len, wl.head_dim
    assert d == 128 and Hq % Hkv == 0
    g = Hq // Hkv
    if plants is None:
        plants = draw_plants(wl, seed)
    crng = np.random.Generator(np.random.Philox(key=[seed, 0x51ED270B]))

    a = c = float(np.sqrt(BETA * np.sqrt(d)))
    diag_gain = np.float32(BETA * np.sqrt(d) / PLANT_LO)

    # every head draws from its own Philox stream, so heads can be generated in parallel
    def base(stream):
        r = np.random.Generator(np.random.Philox(key=[seed, stream]))
        return r.standard_normal((N, d), dtype=np.float32)

    workers = max(1, min(16, os.cpu_count() or 1))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        K0 = np.stack(list(ex.map(lambda kv: base(1000 + kv), range(Hkv))))
        V = np.stack(list(ex.map(lambda kv: base(2000 + kv), range(Hkv))))
    K0[:, :, PLANT_LO:] = 0.0
    K = K0.copy()
    Qb = np.empty((Hq, N, d), dtype=np.uint16)

    def code():
        u = crng.standard_normal(d - CODE_LO).astype(np.float32)
        return u / np.float32(np.linalg.norm(u))

    # K-side plants first (shared by the query heads of a KV group) ...
    qside = []
    for h, p in enumerate(plants):
        kv = h // g
        ch = PLANT_LO + (h % 4)
        ops = {"ch": None, "codes": []}
        planted_keys = np.concatenate([p.sinks, p.cols]).astype(np.int64)
        if planted_keys.size:
            K[kv, planted_keys, ch] = a
            ops["ch"] = ch
        if p.window:
            half = max(p.window // 2, 1)
            nblk = (N + half - 1) // half
            us = [code() for _ in range(nblk)]
            for cb in range(nblk):
                K[kv, cb * half:(cb + 1) * half, CODE_LO:] += np.float32(a) * us[cb]
            ops["window"] = (half, us)
        for (R, C) in p.hot:
            u = code()
            hb = p.hot_block
            K[kv, C * hb:(C + 1) * hb, CODE_LO:] += np.float32(a) * u
            ops["codes"].append((int(R), u))
        qside.append(ops)

    # ... then each query head
    def make_q(h):
        p = plants[h]
        kv = h // g
        q = base(3000 + h)
        q[:, PLANT_LO:] = 0.0
        ops = qside[h]
        if ops["ch"] is not None:
            q[:, ops["ch"]] = c
        for o in p.offs:
            o = int(o)
            q[o:, :PLANT_LO] += diag_gain * K0[kv, :N - o, :PLANT_LO]
        if "window" in ops:
            half, us = ops["window"]
            for cb in range(len(us)):
                sl = slice(cb * half, (cb + 1) * half)
                q[sl, CODE_LO:] += np.float32(c) * us[cb]
                if cb > 0:
                    q[sl, CODE_LO:] += np.float32(c) * us[cb - 1]
        for (R, u) in ops["codes"]:
            hb = p.hot_block
            q[R * hb:(R + 1) * hb, CODE_LO:] += np.float32(c) * u
        Qb[h] = f32_to_bf16_bits(q)

    with ThreadPoolExecutor(max_workers=workers) as ex:
        list(ex.map(make_q, range(Hq)))

    return {
        "Q": Qb,
        "K": f32_to_bf16_bits(K),
        "V": f32_to_bf16_bits(V),
        "plants": plants,
        "workload": wl,
        "seed": seed,
    }


def random_qkv(Hq: int, Hkv: int, N: int, d: int, seed: int, std: float = 1.0):
    """Unstructured bf16 N(0,std^2) Q/K/V (uint16 bits) for small tests."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 7]))
    Q = rng.standard_normal((Hq, N, d), dtype=np.float32) * np.float32(std)
    K = rng.standard_normal((Hkv, N, d), dtype=np.float32) * np.float32(std)
    V = rng.standard_normal((Hkv, N, d), dtype=np.float32)
    return f32_to_bf16_bits(Q), f32_to_bf16_bits(K), f32_to_bf16_bits(V)
