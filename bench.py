#!/usr/bin/env python3
"""Benchmark of the sparse prefill attention hot path on one MI355X.

A step is one pass of the whole path (sa_estimate_patterns -> sa_build_index ->
sa_sparse_prefill) over the Q/K/V of one synthetic attention layer that is
already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--layers L]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
PREWARM_S = 0.25              # untimed load before the W warm-up steps (clock ramp of an idle device)
PAPER_TTFT_S = {"cfg3": 11.1209, "cfg5": 36.3091}   # whole-model TTFT on 2x A5000 (Table 1): context only


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(orc, data, wl, bud, sample_rows):
    """The oracle as it stands, timed on the host: estimator and index in full, masked
    attention on `sample_rows` seeded rows per head, scaled to all rows."""
    import numpy as np

    N, b, w = wl.seq_len, wl.block, wl.last_q
    t0 = time.perf_counter()
    v, s, blk = orc.estimate(data["Q"], data["K"], b, w)
    t1 = time.perf_counter()
    ix = orc.build_index(v.astype(np.float32), s.astype(np.float32), blk.astype(np.float32), N, b, w, bud)
    t2 = time.perf_counter()
    rng = np.random.Generator(np.random.Philox(key=[wl.seed, 99]))
    rows = np.sort(rng.choice(N, size=min(sample_rows, N), replace=False)).astype(np.int32)
    orc.masked_rows(data["Q"], data["K"], data["V"], b, ix, rows=rows)
    t3 = time.perf_counter()
    scale = N / rows.size
    total = (t1 - t0) + (t2 - t1) + (t3 - t2) * scale
    return {
        "value": round(total * 1e3, 1), "unit": "ms/layer", "cores": orc.num_threads(), "kind": "oracle",
        "sample": (f"fp64 oracle: estimator {1e3 * (t1 - t0):.0f} ms and index {1e3 * (t2 - t1):.0f} ms in full; "
                   f"masked attention on {rows.size} seeded rows per head took {1e3 * (t3 - t2):.0f} ms, "
                   f"scaled x{scale:.0f} to all {N} rows"),
    }


def run_workload(name, steps, warmup, layers, with_cpu, sample_rows, with_dense=False, block_select=0,
                 diagonal_select=0, prewarm_s=PREWARM_S, lazy_block_map=0, force_pattern=None, plain=False):
    import numpy as np
    import torch

    import paper_2412_06198_amd as sa
    from harness import gen

    wl = gen.WORKLOADS[name]
    N, b, w, Hq, Hkv, d = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    dev = torch.device("cuda:0")
    ov = None if force_pattern is None else [int(force_pattern)] * Hq   # every head forced to one pattern
    ses = sa.Session(Hq, Hkv, N, b, w, keep=wl.keep, block_select=block_select, diagonal_select=diagonal_select,
                     lazy_block_map=lazy_block_map)

    def up(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    resident, first = [], None
    for l in range(layers):
        t = time.perf_counter()
        data = gen.generate(wl, seed=wl.seed + l)
        if first is None:
            first = data
        resident.append((up(data["Q"]), up(data["K"]), up(data["V"]), [p.pattern for p in data["plants"]]))
        log(f"[{name}] layer {l}: generated + uploaded in {time.perf_counter() - t:.1f} s")
    O = torch.empty_like(resident[0][0])
    torch.cuda.synchronize()

    def step(l, ev=None):
        Q, K, V, _ = resident[l % layers]
        if ev: ev[0].record()
        ses.estimate(Q, K)
        if ev: ev[1].record()
        ses.build_index(ov)
        if ev: ev[2].record()
        ses.prefill(Q, K, V, O)
        if ev: ev[3].record()

    # the device leaves its idle clocks only after some tens of milliseconds of load: bring it to
    # the steady state first (untimed, like the W warm-up steps that follow)
    t_pre, n_pre = time.perf_counter(), 0
    while time.perf_counter() - t_pre < prewarm_s:
        step(n_pre)
        n_pre += 1
        if n_pre % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, evs[i])
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ph = np.array([[e[k].elapsed_time(e[k + 1]) for k in range(3)] for e in evs])
    t_est, t_idx, t_attn = ph.mean(0)
    log(f"[{name}] ms/step wall {wall_ms / steps:.3f}; estimate {t_est:.3f} index {t_idx:.3f} attention {t_attn:.3f}")

    # every resident layer once more, each with its own events: the per-layer spread of the sweep
    # (the K timed steps above cycle the layers from the first one and cover them all only when
    # K >= layers)
    sweep = None
    if layers > 2 and not plain:
        evl = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(layers)]
        for l in range(layers):
            step(l, evl[l])
        torch.cuda.synchronize()
        pl = np.array([[e[k].elapsed_time(e[k + 1]) for k in range(3)] for e in evl])
        tot = pl.sum(1)
        sweep = {"layers": layers, "ms_per_layer_mean": float(tot.mean()), "ms_per_layer_p95": float(np.percentile(tot, 95)),
                 "ms_per_layer_min": float(tot.min()), "ms_per_layer_max": float(tot.max()),
                 "attention_ms_mean": float(pl[:, 2].mean()), "attention_ms_p95": float(np.percentile(pl[:, 2], 95)),
                 "estimate_ms_mean": float(pl[:, 0].mean()), "index_ms_mean": float(pl[:, 1].mean()),
                 "ms_per_layer": [round(float(x), 4) for x in tot]}
        # the first two layers alone, cycled, with all layers still resident: separates what the
        # seeds of the other layers cost from what the larger resident set costs
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for i in range(4):
            step(i % 2)
        e0.record()
        for i in range(16):
            step(i % 2)
        e1.record()
        torch.cuda.synchronize()
        sweep["first_two_layers_cycled_ms_per_layer"] = e0.elapsed_time(e1) / 16
        log(f"[{name}] {layers}-layer sweep: mean {tot.mean():.3f} p95 {np.percentile(tot, 95):.3f} min {tot.min():.3f} "
            f"max {tot.max():.3f} ms/layer; layers 0-1 cycled alone {sweep['first_two_layers_cycled_ms_per_layer']:.3f}")

    # the same step with estimator and index builder as one call (interleaved on two streams)
    def step1(l, ev=None):
        Q, K, V, _ = resident[l % layers]
        if ev: ev[0].record()
        ses.estimate_and_index(Q, K, ov)
        if ev: ev[1].record()
        ses.prefill(Q, K, V, O)
        if ev: ev[2].record()

    wall1_ms, ph1 = float('nan') * steps, np.array([float('nan'), float('nan')])
    if not plain:    # --plain runs only the three-call loop (kernel traces whose averages must match the timed loop)
        for i in range(warmup):
            step1(i)
        torch.cuda.synchronize()
        evs1 = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            step1(i, evs1[i])
        torch.cuda.synchronize()
        wall1_ms = (time.perf_counter() - t0) * 1e3
        ph1 = np.array([[e[k].elapsed_time(e[k + 1]) for k in range(2)] for e in evs1]).mean(0)
        log(f"[{name}] one-call form{' (block map for the Block-Cluster heads only)' if lazy_block_map else ''}: ms/step wall {wall1_ms / steps:.3f}; estimate+index {ph1[0]:.3f} attention {ph1[1]:.3f}")

    # the three-call step recorded once per resident layer into a HIP graph and replayed
    # (a side figure: a failure here must not cost the benchmark line)
    wallg_ms = None
    try:
        if plain:
            raise RuntimeError('--plain')
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graphs = []
        for l in range(min(layers, max(steps, 1))):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                step(l)
            graphs.append(g)
        for i in range(warmup):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        wallg_ms = (time.perf_counter() - t0) * 1e3
        log(f"[{name}] graph replay of the three calls: ms/step wall {wallg_ms / steps:.3f}")
        del graphs
    except Exception as e:  # noqa: BLE001
        log(f"[{name}] graph replay skipped: {e!r}")
        torch.cuda.synchronize()

    # work accounting (untimed): tiles multiplied and kept pairs per layer, pattern choices
    tiles, kept, confusion = [], [], np.zeros((3, 3), int)
    for l in range(layers):
        Q, K, V, planted = resident[l]
        ses.estimate(Q, K)
        ses.build_index(ov)
        c = ses.prefill_counted(Q, K, V, O)
        tiles.append(c[0]); kept.append(c[1])
        for pp, ch in zip(planted, ses.pattern.cpu().tolist()):
            if pp >= 0:
                confusion[pp, ch] += 1
    # The attention kernel's two regimes on layer 0: the tile loop alone (the same index with its
    # diagonal lists emptied) against its MFMA roof, and what the diagonals add against the memory
    # roof (each (wave, diagonal) tile fetches 32 K rows and 32 V rows that nothing else uses).
    attn_phases = None
    if not plain:
        Q, K, V, _ = resident[0]
        ses.estimate(Q, K)
        ses.build_index(ov)
        c_full = ses.prefill_counted(Q, K, V, O)
        saved_n_offs = ses.n_offs.clone()

        def time_prefill(n=6):
            for _ in range(2):
                ses.prefill(Q, K, V, O)
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            for _ in range(n):
                ses.prefill(Q, K, V, O)
            a1.record()
            torch.cuda.synchronize()
            return a0.elapsed_time(a1) / n

        t_full = time_prefill()
        ses.n_offs.zero_()
        c_tile = ses.prefill_counted(Q, K, V, O)
        t_tile = time_prefill()
        ses.n_offs.copy_(saved_n_offs)
        diag_tiles = c_full[0] - c_tile[0]                 # one 32-key tile per (wave, diagonal)
        diag_bytes = diag_tiles * 32 * 2 * d * 2           # 32 K rows + 32 V rows of d bf16 each
        f_tile_loop = 4.0 * d * c_tile[0] * 32 * 32
        t_diag = max(t_full - t_tile, 1e-6)
        attn_phases = {
            "layer": 0, "attention_ms": t_full,
            "tile_loop": {"ms": t_tile, "flop_on_tiles": f_tile_loop, "TFLOPs_on_tiles": f_tile_loop / t_tile / 1e9,
                          "frac_of_bf16_peak": f_tile_loop / t_tile / 1e9 / PEAK_BF16_TFLOPS,
                          "how": "same index with n_offs = 0 (no diagonal phase)"},
            "diagonals": {"ms": t_diag, "bytes": diag_bytes, "GBps": diag_bytes / t_diag / 1e6,
                          "frac_of_hbm_peak": diag_bytes / t_diag / 1e6 / PEAK_HBM_GBS,
                          "kept_pairs": c_full[1] - c_tile[1],
                          "how": "difference to the full call; bytes = 32 K + 32 V rows per (wave, diagonal) tile"},
        }
        log(f"[{name}] attention {t_full:.3f} ms = tile loop {t_tile:.3f} ms ({attn_phases['tile_loop']['TFLOPs_on_tiles']:.0f} TFLOP/s on tiles) "
            f"+ diagonals {t_diag:.3f} ms ({diag_bytes / 1e9:.2f} GB, {attn_phases['diagonals']['GBps']:.0f} GB/s)")
    f_mask = 4.0 * d * float(np.mean(kept))
    f_tiles = 4.0 * d * float(np.mean(tiles)) * 32 * 32   # counter unit: one 32 x 32 sub-tile
    f_dense = 4.0 * d * Hq * N * (N + 1) / 2.0
    nb = N // b
    est_bytes = 2 * Hkv * N * d + 2 * Hq * N * d + 2 * Hq * w * d + 8 * Hq * N + 4 * Hq * nb * nb
    # what a plain device-to-device copy of 1 GiB moves on this machine (read + write): the rate a
    # streaming kernel can be held against, beside the published peak
    cs = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    cd = torch.empty_like(cs)
    for _ in range(2):
        cd.copy_(cs)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        cd.copy_(cs)
    c1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * (1 << 30) * 5 / c0.elapsed_time(c1) / 1e6
    del cs, cd
    res = {
        "workload": name, "ms_per_step": wall_ms / steps, "prewarm_steps_untimed": n_pre,
        "one_call_estimate_and_index": None if plain else {"ms_per_step": wall1_ms / steps,
                                                             "estimate_and_index": float(ph1[0]), "attention": float(ph1[1])},
        "graph_replay_ms_per_step": None if wallg_ms is None else wallg_ms / steps,
        "phases_ms": {"estimate": float(t_est), "index": float(t_idx), "attention": float(t_attn),
                      "attention_p95": float(np.percentile(ph[:, 2], 95))},
        "tflops": {"kept": f_mask / t_attn / 1e9, "tiles": f_tiles / t_attn / 1e9,
                   "dense_equivalent": f_dense / (wall_ms / steps) / 1e9},
        "flop": {"kept": f_mask, "tiles": f_tiles, "dense": f_dense},
        "kept_fraction_of_causal": float(np.mean(kept)) / (Hq * N * (N + 1) / 2.0),
        "mfma_frac_of_peak_on_tiles": f_tiles / t_attn / 1e9 / PEAK_BF16_TFLOPS,
        "estimator": {"algorithmic_bytes": est_bytes, "GBps": est_bytes / t_est / 1e6,
                      "frac_of_hbm_peak": est_bytes / t_est / 1e6 / PEAK_HBM_GBS,
                      "device_copy_GBps_same_run": copy_gbps},
        "attention_phases": attn_phases,
        "layer_sweep": sweep,
        "pattern_confusion_planted_x_chosen": confusion.tolist(),
        "paper_context": {"ttft_s_whole_model_2xA5000": PAPER_TTFT_S.get(name)},
    }
    if with_dense:
        # the same kernel on an all-keys index (Triangular with the band as wide as the sequence):
        # plain causal attention, the clean figure for the tile loop itself
        Q, K, V, _ = resident[0]
        dn = sa.Session(Hq, Hkv, N, b, w, keep=wl.keep, local_blocks=nb, k_blocks=nb * (nb + 1) // 2)
        dn.estimate(Q, K)
        dn.build_index([sa.SA_TRIANGULAR] * Hq)
        for _ in range(2):
            dn.prefill(Q, K, V, O)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(4):
            dn.prefill(Q, K, V, O)
        e1.record()
        torch.cuda.synchronize()
        t_dense = e0.elapsed_time(e1) / 4
        res["dense_all_keys_index"] = {"ms": t_dense, "TFLOPs_causal": f_dense / t_dense / 1e9,
                                       "frac_of_bf16_peak": f_dense / t_dense / 1e9 / PEAK_BF16_TFLOPS}
        log(f"[{name}] dense (all-keys index) {t_dense:.3f} ms = {f_dense / t_dense / 1e9:.0f} TFLOP/s")
        dn.close()
    if with_cpu:
        from oracle import oracle as orc
        bud = orc.default_budgets(N, b, wl.keep)
        bud.block_select = block_select
        bud.diagonal_select = diagonal_select
        res["cpu_baseline"] = cpu_baseline(orc, first, wl, bud, sample_rows)
        log(f"[{name}] cpu_baseline {res['cpu_baseline']}")
    ses.close()
    del resident, O
    torch.cuda.empty_cache()
    return res


def run_block_rules(name, steps):
    """The readings of Alg. 3's TopKBlocks side by side on one layer: one top-k over the whole
    block map, the same fraction of every row, and one top-k on the row-normalised key.  Error = Frobenius distance of the sparse
    output to the all-keys output of the same kernel, over the Block-Cluster heads."""
    import numpy as np
    import torch

    import paper_2412_06198_amd as sa
    from harness import gen

    wl = gen.WORKLOADS[name]
    N, b, w, Hq, Hkv, d = wl.seq_len, wl.block, wl.last_q, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    nb = N // b
    dev = torch.device("cuda:0")
    data = gen.generate(wl)

    def up(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    Q, K, V = up(data["Q"]), up(data["K"]), up(data["V"])
    outs, res = {}, {"workload": name}
    for label, kw in (("all_keys", dict(local_blocks=nb, k_blocks=nb * (nb + 1) // 2)),
                      ("global", dict(block_select=0)), ("per_row", dict(block_select=1)),
                      ("row_normalised", dict(block_select=2))):
        ses = sa.Session(Hq, Hkv, N, b, w, keep=wl.keep, **kw)
        O = torch.empty_like(Q)
        ov = [sa.SA_TRIANGULAR] * Hq if label == "all_keys" else None
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        tot = np.zeros(3)
        for i in range(steps + 1):
            ev[0].record(); ses.estimate(Q, K)
            ev[1].record(); ses.build_index(ov)
            ev[2].record(); ses.prefill(Q, K, V, O)
            ev[3].record()
            torch.cuda.synchronize()
            if i:
                tot += [ev[k].elapsed_time(ev[k + 1]) for k in range(3)]
        tiles, kept = ses.prefill_counted(Q, K, V, O)
        torch.cuda.synchronize()
        outs[label] = (O, ses.pattern.cpu().numpy().copy(), ses.rowptr[:, nb].cpu().numpy().copy())
        res[label] = {"phases_ms": dict(zip(("estimate", "index", "attention"), (tot / steps).round(4).tolist())),
                      "kept_pairs": int(kept), "tiles": int(tiles)}
        ses.close()
    pat = outs["global"][1]
    assert (pat == outs["per_row"][1]).all() and (pat == outs["row_normalised"][1]).all()
    bc = np.nonzero(pat == sa.SA_BLOCK_CLUSTER)[0]
    ref = outs["all_keys"][0].float()
    for label in ("global", "per_row", "row_normalised"):
        diff = (outs[label][0].float() - ref)[torch.from_numpy(bc).to(dev)]
        err = torch.linalg.vector_norm(diff.double(), dim=(1, 2)).cpu().numpy()
        res[label]["block_cluster_heads"] = bc.tolist()
        res[label]["blocks_per_bc_head"] = outs[label][2][bc].tolist()
        res[label]["frobenius_error_per_bc_head"] = err.round(3).tolist()
        res[label]["frobenius_error_mean"] = float(err.mean())
        log(f"[{name}] {label}: {res[label]['phases_ms']} mean error over {len(bc)} Block-Cluster heads {err.mean():.3f}")
    print(json.dumps({"block_rules": res}))


def run_sweep(steps):
    """Dense (all-keys index) against sparse (estimate + index + attention) per layer, 4K ... 128K:
    where the method starts to pay on this GPU (the paper puts that threshold at 16K-32K tokens
    on its own hardware; Experimental Results, TTFT table and its discussion)."""
    import numpy as np
    import torch

    import paper_2412_06198_amd as sa
    from harness import gen

    def up(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()

    rows = []
    for N, b, keep in ((4096, 64, 0.10), (8192, 64, 0.125), (16384, 64, 0.125), (32768, 64, 0.06),
                       (65536, 128, 0.04), (131072, 128, 0.03)):
        wl = gen.scaled(gen.WORKLOADS["cfg3"], name=f"sweep{N}", seq_len=N, block=b, keep=keep, seed=7000 + N,
                        hot_block=b)
        data = gen.generate(wl)
        Hq, Hkv, w, d = wl.n_q_heads, wl.n_kv_heads, wl.last_q, wl.head_dim
        Q, K, V = up(data["Q"]), up(data["K"]), up(data["V"])
        O = torch.empty_like(Q)
        nb = N // b
        res = {}
        for kind in ("sparse", "dense"):
            if kind == "sparse":
                ses = sa.Session(Hq, Hkv, N, b, w, keep=keep)
            else:  # every causal block kept: Triangular with the band as wide as the sequence
                ses = sa.Session(Hq, Hkv, N, b, w, keep=keep, local_blocks=nb, k_blocks=nb * (nb + 1) // 2)

            def step():
                if kind == "sparse":
                    ses.estimate(Q, K)
                    ses.build_index(None)
                else:
                    pass
                ses.prefill(Q, K, V, O)

            if kind == "dense":
                ses.estimate(Q, K)
                ses.build_index([sa.SA_TRIANGULAR] * Hq)   # the index is built once, outside the timing
            n = steps if N <= 32768 or kind == "sparse" else max(2, steps // 4)
            for _ in range(2):
                step()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                step()
            e1.record()
            torch.cuda.synchronize()
            res[kind] = e0.elapsed_time(e1) / n
            if kind == "sparse":
                # the same step recorded once into a HIP graph and replayed: what the ten small
                # launches of the index builder cost on the host side at short sequences
                res["sparse_graph"] = float("nan")
                try:
                    side = torch.cuda.Stream()
                    side.wait_stream(torch.cuda.current_stream())
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph, stream=side):
                        step()
                    for _ in range(2):
                        graph.replay()
                    torch.cuda.synchronize()
                    e0.record()
                    for _ in range(n):
                        graph.replay()
                    e1.record()
                    torch.cuda.synchronize()
                    res["sparse_graph"] = e0.elapsed_time(e1) / n
                    del graph
                except Exception as e:  # noqa: BLE001
                    log(f"[sweep] graph replay skipped: {e!r}")
                    torch.cuda.synchronize()
            ses.close()
        f_dense = 4.0 * d * Hq * N * (N + 1) / 2.0
        rows.append({"seq_len": N, "block": b, "keep": keep, "sparse_ms": round(res["sparse"], 4),
                     "sparse_graph_replay_ms": round(res["sparse_graph"], 4),
                     "dense_ms": round(res["dense"], 4), "speedup": round(res["dense"] / res["sparse"], 3),
                     "dense_TFLOPs": round(f_dense / res["dense"] / 1e9, 1)})
        log(f"[sweep] N={N}: sparse {res['sparse']:.3f} ms (graph replay {res['sparse_graph']:.3f}), dense {res['dense']:.3f} ms "
            f"({rows[-1]['dense_TFLOPs']} TFLOP/s), ratio {rows[-1]['speedup']}")
        del Q, K, V, O
        torch.cuda.empty_cache()
    print(json.dumps({"sweep": "dense (all-keys index) vs sparse path per layer, Hq=32 Hkv=8 d=128, "
                               "planted mix 25/50/25", "rows": rows}))


def run_search(N, with_cpu):
    """Offline pattern search (Kernel-Aware Sparse Pattern Search Algorithm, Alg. 1) on one GQA
    group (planted Triangular, Interval-Slash, Interval-Slash, Block-Cluster heads): seconds per
    head, what it chose, and the oracle of the same search timed on a small head beside it."""
    import numpy as np
    import torch

    import paper_2412_06198_amd as sa
    from harness import gen

    def up(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()

    b = 64 if N <= 32768 else 128
    wl = gen.scaled(gen.WORKLOADS["cfg3"], name=f"search{N}", seq_len=N, block=b, n_q_heads=4, n_kv_heads=1,
                    hot_block=b, seed=8000 + N)
    data = gen.generate(wl)
    Q, K, V = up(data["Q"]), up(data["K"]), up(data["V"])
    ses = sa.Session(4, 1, N, b, wl.last_q, keep=wl.keep)
    ses.estimate(Q, K)
    torch.cuda.synchronize()
    target = int(N * (N + 1) // 2 * wl.keep)
    eps = target // 100
    ses.search_patterns(Q, K, V, target, eps)          # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    res = ses.search_patterns(Q, K, V, target, eps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    out = {"search": f"Alg. 1 on one GQA group, N={N} block={b}, target {wl.keep} of the causal pairs +-1%",
           "seconds_per_head": round(dt / 4, 4), "planted": [int(pl.pattern) for pl in data["plants"]],
           "chosen": [r["pattern"] for r in res], "param": [r["param"] for r in res],
           "pairs_over_target": [[round(x / target, 4) for x in r["pairs"]] for r in res],
           "err": [[round(x, 3) for x in r["err"]] for r in res]}
    log(f"[search] N={N}: {dt / 4:.3f} s per head, planted {out['planted']} chosen {out['chosen']}")
    ses.close()
    if with_cpu:
        from oracle import oracle as orc
        from oracle import search as osr
        n = 2048
        wls = gen.scaled(wl, seq_len=n, block=64, n_q_heads=1, window=min(wl.window, 256), hot_block=64)
        ds = gen.generate(wls)
        v, s_, blk = [x.astype(np.float32) for x in orc.estimate(ds["Q"], ds["K"], 64, wls.last_q)]
        tg = int(n * (n + 1) // 2 * 0.2)
        t0 = time.perf_counter()
        osr.search_patterns(ds["Q"], ds["K"], ds["V"], v, s_, blk, 64, wls.last_q, 1, tg, tg // 100)
        out["cpu_baseline"] = {"value": round(time.perf_counter() - t0, 3), "unit": "s per head", "cores": orc.num_threads(),
                               "kind": "oracle", "sample": f"fp64 oracle of the same search on one head of {n} tokens"}
    print(json.dumps(out))


def run_decode(name, steps):
    """One decode step over the prefill index of a benchmark workload (the query of the next
    token): microseconds per step for all heads and the HBM rate on the K and V rows it lists."""
    import numpy as np
    import torch

    import paper_2412_06198_amd as sa
    from harness import gen

    def up(bits):
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()

    wl = gen.WORKLOADS[name]
    data = gen.generate(wl)
    Hq, Hkv, N, b, d = wl.n_q_heads, wl.n_kv_heads, wl.seq_len, wl.block, wl.head_dim
    pad = 64                                   # room for generated keys behind the prompt
    Q = up(data["Q"])
    K = torch.zeros((Hkv, N + pad, d), dtype=torch.bfloat16, device="cuda")
    V = torch.zeros_like(K)
    K[:, :N], V[:, :N] = up(data["K"]), up(data["V"])
    K[:, N:], V[:, N:] = K[:, :pad], V[:, :pad]   # stand-ins for the generated tokens' keys and values
    ses = sa.Session(Hq, Hkv, N, b, wl.last_q, keep=wl.keep, kv_head_stride=(N + pad) * d)
    ses.estimate(Q, K)
    ses.build_index(None)
    q = Q[:, N - 1].contiguous()
    o = torch.empty_like(q)
    pos = N + 7
    for _ in range(3):
        ses.decode(q, K, V, pos, o)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        ses.decode(q, K, V, pos, o)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / steps * 1e3
    nb = N // b
    listed = ((ses.rowptr[:, nb] - ses.rowptr[:, nb - 1]).clamp(min=0) * b + ses.n_cols.clamp(min=0) +
              ses.n_offs.clamp(min=0) + (pos - N + 1)).sum().item()
    byt = listed * 2 * d * 2
    out = {"decode": f"one decode step over the prefill index, {name}: Hq={Hq} Hkv={Hkv} N={N} block={b} keep={wl.keep}",
           "us_per_step": round(us, 2), "listed_keys_all_heads": int(listed),
           "roofline": {"bound": "hbm", "kernel": "decode_partial_kernel", "achieved": round(byt / us / 1e3, 1),
                        "peak": 8000.0, "unit": "GB/s", "frac": round(byt / us / 1e3 / 8000.0, 4), "traffic": None},
           "note": "bytes = K and V rows of the listed keys (before the union drops repeats); two launches per step"}
    log(f"[decode] {name}: {us:.1f} us per step, {listed} keys listed, {byt / us / 1e3:.0f} GB/s")
    ses.close()
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg5", help="cfg1..cfg5; cfg5 = 128K tokens, cfg3 = 32K")
    ap.add_argument("--layers", type=int, default=0,
                    help="distinct seeded layers kept resident and cycled by the steps; 0 = 32 for cfg5 (the "
                         "benchmark's 32-layer sweep with independent seeds), 2 otherwise")
    ap.add_argument("--also", default="cfg3", help="second workload reported under 'also' ('' to skip)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--prewarm", type=float, default=PREWARM_S,
                    help="seconds of untimed load before the warm-up steps (0 for counter-collection runs)")
    ap.add_argument("--sample-rows", type=int, default=16384,
                    help="rows per head of the oracle's masked attention in the cpu_baseline leg (about 10 s at 128K)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (reference for HBM byte counters)")
    ap.add_argument("--sweep", action="store_true",
                    help="dense-vs-sparse time per layer from 4K to 128K tokens instead of the benchmark line")
    ap.add_argument("--search", type=int, default=0, metavar="N",
                    help="time the offline pattern search (Alg. 1) on one GQA group of N tokens instead")
    ap.add_argument("--block-select", choices=("global", "row"), default="global",
                    help="how Block-Cluster heads spend k_blocks: one top-k (Alg. 3 read literally) or the same "
                         "fraction of every row block")
    ap.add_argument("--diagonals", choices=("exact", "blocks"), default="exact",
                    help="selected diagonals of Interval-Slash heads element-exact (default) or widened to whole blocks")
    ap.add_argument("--force-pattern", choices=["T", "IS", "BC"], default=None,
                    help="override the pattern rule: every head Triangular, Interval-Slash or Block-Cluster "
                         "(per-pattern timing and counters; not the benchmark's workload)")
    ap.add_argument("--lazy-block-map", action="store_true",
                    help="one-call form: compute the block map only for the heads decided Block-Cluster")
    ap.add_argument("--block-rules", action="store_true",
                    help="compare the two block rules (time, kept pairs, error against all-keys attention) instead")
    ap.add_argument("--plain", action="store_true",
                    help="run only the three-call loop and the work accounting (for kernel traces: the traced "
                         "averages are then those of the timed steps)")
    ap.add_argument("--decode", action="store_true",
                    help="time one decode step over the prefill index of --workload instead")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (heads shard without communication; "
              "no multi-GPU path is built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if a.copy_calibration:
        # a copy kernel of known size: reads 1 GiB, writes 1 GiB per launch
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").random_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 4}}))
        return
    import paper_2412_06198_amd as sa

    sa.library()
    if a.sweep:
        run_sweep(a.steps)
        return
    if a.decode:
        run_decode(a.workload, max(a.steps, 50))
        return
    if a.block_rules:
        run_block_rules(a.workload, a.steps)
        return
    if a.search:
        run_search(a.search, not a.no_cpu_baseline)
        return
    if a.layers <= 0:
        a.layers = 32 if a.workload == "cfg5" else 2
    bsel = 1 if a.block_select == "row" else 0
    fpat = None if a.force_pattern is None else {"T": 0, "IS": 1, "BC": 2}[a.force_pattern]
    dsel = 1 if a.diagonals == "blocks" else 0
    main_res = run_workload(a.workload, a.steps, a.warmup, a.layers, not a.no_cpu_baseline, a.sample_rows,
                            block_select=bsel, diagonal_select=dsel, prewarm_s=a.prewarm,
                            lazy_block_map=int(a.lazy_block_map), force_pattern=fpat, plain=a.plain)
    also = None
    if a.also and a.also != a.workload:
        also = run_workload(a.also, max(a.steps, 20), a.warmup, min(a.layers, 2), False, a.sample_rows,
                            with_dense=True, block_select=bsel, diagonal_select=dsel, prewarm_s=a.prewarm,
                            lazy_block_map=int(a.lazy_block_map), force_pattern=fpat)

    traffic = None
    tp = os.path.join(ROOT, "profiles", f"traffic_{a.workload}.json")
    if os.path.exists(tp):
        traffic = json.load(open(tp)).get("sparse_prefill_kernel_hbm_bytes_per_launch")
    from harness import gen
    wl = gen.WORKLOADS[a.workload]
    # what the attention kernel cannot avoid moving: Q read and O written once, K and V read once
    compulsory = 2 * (2 * wl.n_q_heads * wl.seq_len * wl.head_dim) + 2 * (2 * wl.n_kv_heads * wl.seq_len * wl.head_dim)
    out = {
        "metric": "sparse prefill attention ms/layer (estimate + index + attention)",
        "value": round(main_res["ms_per_step"], 4), "unit": "ms/layer",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(main_res["ms_per_step"], 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{a.workload}: Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} d={wl.head_dim} "
                               f"N={wl.seq_len} block={wl.block} last_q={wl.last_q} keep={wl.keep} "
                               f"layers={a.layers} (seeds {wl.seed}..{wl.seed + a.layers - 1}), "
                               + ("patterns chosen at run time" if fpat is None else f"every head forced to pattern {a.force_pattern}")
                               + (", blocks chosen per row" if bsel else "")
                               + (", diagonals widened to blocks" if dsel else "")},
        "roofline": {"bound": "mfma", "kernel": "sparse_prefill_kernel",
                     "achieved": round(main_res["tflops"]["kept"], 2), "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(main_res["tflops"]["kept"] / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic, "compulsory_bytes": compulsory,
                     "traffic_over_compulsory": None if not traffic else round(traffic / compulsory, 2),
                     "achieved_on_computed_tiles": round(main_res["tflops"]["tiles"], 2),
                     "frac_on_computed_tiles": round(main_res["mfma_frac_of_peak_on_tiles"], 4)},
        "cpu_baseline": main_res.pop("cpu_baseline", None),
        "detail": main_res,
        "also": also,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
