#!/usr/bin/env python3
"""Benchmark of the DIP / DIP-CA hot path on one MI355X.

A step is one decode token through one SwiGLU MLP layer (scores -> top-K -> gathered
up/gate GEMV + SwiGLU -> scores -> top-K -> gathered down GEMV, plus the cache updates in
the DIP-CA configurations), called through the C ABI of libdip.  All inputs are synthetic
and resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4|5] [--ratio R] [--cache-frac C]

The default workload is BASELINE configs[3]: the Phi-3-Medium-shaped stack of 40 bf16 layers,
keep ratio 0.3, DIP-CA with an LRU cache over half of the columns, gamma 0.2.  Steps walk the
stack token-major; exactly --steps of them form a timed block, and the reported time is the
median over --repeats repeats of that block (run back to back until a repeat lasts 20 ms).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
VALU_PEAK_TFLOPS = 157.3  # fp32 vector: 256 compute units x 128 FMA lanes x 2 flops x 2.4 GHz


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000,
                    help="layer-steps per timed block (one token through one MLP layer each)")
    ap.add_argument("--warmup", type=int, default=400, help="untimed layer-steps before the first timed block")
    ap.add_argument("--repeats", type=int, default=5, help="timed repeats; the median is reported")
    ap.add_argument("--min-repeat-ms", type=float, default=20.0,
                    help="a repeat runs the block of --steps steps as many times as it takes to last this long")
    ap.add_argument("--config", type=int, default=4, choices=(2, 3, 4, 5),
                    help="BASELINE config number (1-based); default 4 = configs[3], the Phi-3-Medium-shaped stack")
    ap.add_argument("--policy", default="lru", choices=("lru", "lfu"))
    ap.add_argument("--tokens", type=int, default=512, help="distinct tokens per layer stream (then it wraps)")
    ap.add_argument("--no-fusion", action="store_true",
                    help="launch selection and product apart (two launches per pruning point)")
    ap.add_argument("--no-side-runs", action="store_true",
                    help="skip the LRU/LFU x gamma hit-rate runs and the simulated-mobile figures")
    ap.add_argument("--side-tokens", type=int, default=48)
    ap.add_argument("--ratio", type=float, default=None, help="keep ratio at both pruning points")
    ap.add_argument("--cache-frac", type=float, default=None)
    ap.add_argument("--layers", type=int, default=None,
                    help="distinct weight copies (config 2) or stack depth (configs 3, 4)")
    ap.add_argument("--batch", type=int, default=1, help="rows per step (config 5 only, 1..8)")
    ap.add_argument("--scheme", default="dip", choices=("dip", "glu", "gate", "up"),
                    help="dip: the headline path; glu / gate / up: the sibling schemes that prune on "
                         "(partial) GLU activations, k = keep ratio of d_ff, no cache")
    ap.add_argument("--tiered", action="store_true",
                    help="two-tier residency: the matrices live in pinned host memory, cache-capacity many "
                         "columns of each in HBM slots; misses cross PCIe (use with --gamma 1.0 / 0.2)")
    ap.add_argument("--gamma", type=float, default=None, help="cache-aware penalty (1.0 = plain DIP keys)")
    ap.add_argument("--tune", default=None,
                    help="lanes_per_row,waves,ksplit,unroll override for the gathered GEMV (0 = built-in choice)")
    ap.add_argument("--graph", action="store_true",
                    help="capture a window of steps into a HIP graph and time its replays "
                         "(default: every step's launches are issued from the host)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=24)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) so that a counter "
                         "pass of rocprofv3 can be scaled against it")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="skip the per-kernel HIP-event pass (roofline becomes null)")
    return ap.parse_args()


def measured_traffic(workload: str, ratio: float, shape) -> "int | None":
    """HBM bytes per up/gate launch from the committed rocprofv3 counter summaries
    (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known size), if one was taken
    for this workload and launch shape; otherwise None."""
    import glob
    want = {"workload": workload, "ratio": f"{ratio:g}", "shape": ",".join(str(v) for v in shape)}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "hbm_traffic_*.txt"))):
        for line in open(path):
            if not line.startswith("workload="):
                continue
            kv = dict(tok.split("=", 1) for tok in line.split())
            if all(kv.get(k) == v for k, v in want.items()):
                return int(kv["gemv_upgate_fetch_bytes"]) + int(kv["gemv_upgate_write_bytes"])
    return None


def bench_scheme(a):
    """One token through one layer under GLU, Gate or Up pruning; same JSON fields as the headline."""
    import numpy as np
    import torch

    import paper_2412_01380_amd as D
    from workloads import CONFIGS, layer_weights, layer_weights_split

    torch.cuda.set_device(0)
    cfg = CONFIGS[a.config]
    r = a.ratio if a.ratio is not None else {2: 0.5, 3: 0.3, 4: 0.3, 5: 0.3}[a.config]
    d, f = cfg.d_model, cfg.d_ff
    k = cfg.k_mid(r)
    L = a.layers if a.layers is not None else 8
    n_tok = cfg.n_tokens
    mk = lambda t: (D.Weight(torch.from_numpy(t[0]).cuda(), torch.from_numpy(t[1]).cuda())
                    if isinstance(t, tuple) else D.Weight(torch.from_numpy(t.view(np.int16)).cuda()))
    mlps, host0 = [], None
    for l in range(L):
        if a.scheme == "glu":
            w = layer_weights(d, f, cfg.seed, l, cfg.dtype)
            mlps.append(D.Mlp(mk(w["ug"]), mk(w["d"])))
        else:
            w = layer_weights_split(d, f, cfg.seed, l, cfg.dtype)
            dense, rows = ("g", "u_rows") if a.scheme == "gate" else ("u", "g_rows")
            w = {"dense": w[dense], "rows": w[rows], "d": w["d"]}
            mlps.append(D.MlpSplit(mk(w["dense"]), mk(w["rows"]), mk(w["d"])))
        if l == 0:
            host0 = w
    X = np.stack([cfg.tokens(layer=l, n_tokens=n_tok) for l in range(L)], axis=1)
    Xd = torch.from_numpy(X).cuda()
    Yd = torch.empty(L, d, dtype=torch.float32, device="cuda")
    if a.scheme == "glu":
        ws = torch.empty(D.dip_glu_pruning_forward_workspace_bytes(mlps[0], k), dtype=torch.uint8, device="cuda")
        step = lambda t, l: D.dip_glu_pruning_forward(mlps[l], Xd[t % n_tok, l], k, Yd[l], None, ws)
    else:
        code = D.DIP_GATE_PRUNING if a.scheme == "gate" else D.DIP_UP_PRUNING
        ws = torch.empty(D.dip_partial_pruning_forward_workspace_bytes(mlps[0], k), dtype=torch.uint8, device="cuda")
        step = lambda t, l: D.dip_partial_pruning_forward(mlps[l], code, Xd[t % n_tok, l], k, Yd[l], None, ws)

    def run_pass(t):
        for l in range(L):
            step(t, l)

    passes_w = max(1, (a.warmup + L - 1) // L)
    passes = max(1, (a.steps + L - 1) // L)
    steps = passes * L
    for t in range(passes_w):
        run_pass(t)
    torch.cuda.synchronize()
    launch_mode = "launches issued from the host, step by step"
    warm_steps = passes_w * L
    if not a.graph:
        t0 = time.perf_counter()
        for t in range(passes):
            run_pass(passes_w + t)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    else:
        # The launches of a window of consecutive passes are captured once into a HIP graph
        # (the library only launches kernels on the given stream: no allocation, no memset, no
        # host synchronisation) and the window is replayed: same kernels, same arguments, same
        # order.  Cache state lives in device memory and keeps evolving from replay to replay.
        # Measured gain over host-issued launches: 1-2 % (the kernels are long enough to hide
        # the host's launch path), hence not the default.
        per_pass = 4 * L
        G = max(g for g in range(1, passes + 1) if passes % g == 0 and (g == 1 or g * per_pass <= 8192))
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for t in range(G):
                run_pass(passes_w + t)
        graph.replay()                      # one untimed replay
        torch.cuda.synchronize()
        warm_steps += G * L
        t0 = time.perf_counter()
        for _ in range(passes // G):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        launch_mode = f"HIP graph of {G} pass(es) = {G * L} steps, replayed {passes // G} times"

    bytes_of = (lambda e: e // 2 + (e // 128) * 2) if cfg.dtype == "int4" else (lambda e: e * 2)
    dense_bytes = bytes_of((2 if a.scheme == "glu" else 1) * d * f)
    rows_bytes = 0 if a.scheme == "glu" else bytes_of(k * d)
    down_bytes = bytes_of(k * d)
    total = dense_bytes + rows_bytes + down_bytes
    out = {
        "metric": "DIP MLP decode tokens/s at batch 1 + achieved HBM GB/s vs peak on gathered bytes",
        "value": steps / wall, "unit": "layer-tokens/s", "n_gpus": 1, "steps": steps,
        "warmup": warm_steps, "ms_per_step": wall / steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"launch": launch_mode, "workload": f"{a.scheme} pruning (Sec. 3.2) on the MLP shape of BASELINE configs[{a.config - 1}]: "
                               f"{cfg.name}, d_model={d}, d_ff={f}, {cfg.dtype} weights, batch 1, k={k} of d_ff kept, "
                               f"{L} distinct weight copies visited round-robin",
                   "inputs": cfg.inputs, "weights_dtype": cfg.dtype, "weight_bytes_per_step": total},
        "end_to_end_GBps": total * steps / wall / 1e9,
    }
    kinds = {"select_in": 0, "gemv_upgate": 1, "select_mid": 2, "gemv_down": 3, "gemv_dense": 4, "rowdot": 5}
    n_prof = min(passes, max(1, 1024 // L))
    D.dip_profile_enable(5 * L * n_prof + 16)
    for t in range(n_prof):
        run_pass(passes_w + passes + t)
    torch.cuda.synchronize()
    prof = {kname: D.dip_profile_read(i) for kname, i in kinds.items()}
    D.dip_profile_disable()
    out["kernels_us"] = {kname: v[0] / v[1] * 1e3 for kname, v in prof.items() if v[1]}
    main_kind, main_bytes = ("gemv_upgate", dense_bytes) if a.scheme == "glu" else ("gemv_dense", dense_bytes)
    ms, n = prof[main_kind]
    ach = main_bytes / (ms / n * 1e-3) / 1e9
    out["roofline"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": ach / HBM_PEAK_GBS, "traffic": None,
                       "kernel": "gemv_kernel (dense first product)", "algorithmic_bytes_per_launch": main_bytes,
                       "avg_launch_us": ms / n * 1e3, "launches": n}
    if prof["rowdot"][1]:
        ms, n = prof["rowdot"]
        out["roofline_rowdot"] = {"achieved": rows_bytes / (ms / n * 1e-3) / 1e9,
                                  "algorithmic_bytes_per_launch": rows_bytes, "avg_launch_us": ms / n * 1e3}
    ms, n = prof["gemv_down"]
    out["roofline_down"] = {"achieved": down_bytes / (ms / n * 1e-3) / 1e9,
                            "algorithmic_bytes_per_launch": down_bytes, "avg_launch_us": ms / n * 1e3}
    if not a.no_cpu_baseline:
        from oracle import dip_oracle as O
        nt = a.cpu_sample_tokens
        c0, w0t = time.process_time(), time.perf_counter()
        for t in range(nt):
            if a.scheme == "glu":
                O.glu_pruning_forward(host0["ug"], host0["d"], X[t % n_tok, 0], k)
            else:
                O.partial_pruning_forward(a.scheme, host0["dense"], host0["rows"], host0["d"], X[t % n_tok, 0], k)
        wall_o, cpu_o = time.perf_counter() - w0t, time.process_time() - c0
        out["cpu_baseline"] = {"value": nt / wall_o, "unit": out["unit"],
                               "cores": max(1, int(round(cpu_o / wall_o))), "kind": "oracle",
                               "sample": f"{nt} tokens through layer 0 of the same workload ({wall_o:.1f} s wall)"}
    print(json.dumps(out))


def bench_tiered(a):
    """DIP-CA with misses that are really slow: per step, the columns a cache update inserts are
    copied host -> HBM and the misses that bypass the cache are read over PCIe by the product."""
    import numpy as np
    import torch

    import paper_2412_01380_amd as D
    from workloads import CONFIGS, layer_weights

    torch.cuda.set_device(0)
    cfg = CONFIGS[a.config]
    assert cfg.dtype != "int4", "tiers hold f32 / bf16 matrices"
    r = a.ratio if a.ratio is not None else 0.3
    frac = a.cache_frac if a.cache_frac is not None else 0.5
    gamma = a.gamma if a.gamma is not None else cfg.gamma
    d, f = cfg.d_model, cfg.d_ff
    k_in, k_mid = cfg.k_in(r), cfg.k_mid(r)
    C_in, C_mid = int(np.floor(frac * d + 0.5)), int(np.floor(frac * f + 0.5))
    L = a.layers if a.layers is not None else 4
    n_tok = cfg.n_tokens

    def pinned(arr):
        t = torch.from_numpy(arr.view(np.int16))
        p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        p.copy_(t)
        return p

    mlps, cins, cmids = [], [], []
    for l in range(L):
        w = layer_weights(d, f, cfg.seed, l, cfg.dtype)
        tu, td = D.TieredWeight(pinned(w["ug"]), C_in), D.TieredWeight(pinned(w["d"]), C_mid)
        ci, cm = D.Cache(d, C_in), D.Cache(f, C_mid)
        for tw, c in ((tu, ci), (td, cm)):
            D.dip_cache_init(c)
            D.dip_tier_init(tw, c, torch.empty(max(256, D.dip_tier_init_workspace_bytes(tw)), dtype=torch.uint8, device="cuda"))
        mlps.append(D.TieredMlp(tu, td)); cins.append(ci); cmids.append(cm)
        del w
    X = np.stack([cfg.tokens(layer=l, n_tokens=n_tok) for l in range(L)], axis=1)
    Xd = torch.from_numpy(X).cuda()
    Yd = torch.empty(L, d, dtype=torch.float32, device="cuda")
    ws = torch.empty(D.dip_tiered_mlp_forward_workspace_bytes(mlps[0], k_in, k_mid), dtype=torch.uint8, device="cuda")

    def run_pass(t):
        for l in range(L):
            D.dip_tiered_mlp_forward(mlps[l], Xd[t % n_tok, l], k_in, k_mid, cins[l], cmids[l], gamma, Yd[l], None, ws)

    def lookups():
        mi = [c.meta_host() for c in cins]
        mm = [c.meta_host() for c in cmids]
        return (sum(m["cum_hits"] for m in mi), sum(m["cum_lookups"] for m in mi),
                sum(m["cum_hits"] for m in mm), sum(m["cum_lookups"] for m in mm))

    passes_w = max(1, (a.warmup + L - 1) // L)
    passes = max(1, (a.steps + L - 1) // L)
    steps = passes * L
    for t in range(passes_w):
        run_pass(t)
    torch.cuda.synchronize()
    h0 = lookups()
    t0 = time.perf_counter()
    for t in range(passes):
        run_pass(passes_w + t)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    h1 = lookups()
    hit_in, look_in, hit_mid, look_mid = (b - a_ for a_, b in zip(h0, h1))
    row_ug, row_d = 2 * f * 2, d * 2
    pcie = (look_in - hit_in) * row_ug + (look_mid - hit_mid) * row_d
    gathered = cfg.gathered_bytes(r)
    D.dip_profile_enable(8 * L * min(passes, 64) + 16)
    for t in range(min(passes, 64)):
        run_pass(passes_w + passes + t)
    torch.cuda.synchronize()
    kinds = {"select_in": 0, "gemv_upgate": 1, "select_mid": 2, "gemv_down": 3, "tier_fill": 6}
    prof = {kname: D.dip_profile_read(i) for kname, i in kinds.items()}
    D.dip_profile_disable()
    ug_ms, ug_n = prof["gemv_upgate"]
    ug_bytes = 2 * k_in * f * 2
    ach = ug_bytes / (ug_ms / ug_n * 1e-3) / 1e9
    out = {
        "metric": "DIP MLP decode tokens/s at batch 1 + achieved HBM GB/s vs peak on gathered bytes",
        "value": steps / wall, "unit": "layer-tokens/s", "n_gpus": 1, "steps": steps, "warmup": passes_w * L,
        "ms_per_step": wall / steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"two-tier residency on the MLP shape of BASELINE configs[{a.config - 1}]: {cfg.name}, "
                               f"d_model={d}, d_ff={f}, {cfg.dtype} weights in pinned host memory, "
                               f"HBM slot cache frac {frac} (C_in={C_in}, C_mid={C_mid}), LRU, gamma {gamma}, "
                               f"keep ratio {r} (k_in={k_in}, k_mid={k_mid}), batch 1, {L} layers round-robin",
                   "inputs": cfg.inputs, "weights_dtype": cfg.dtype, "gathered_bytes_per_step": gathered},
        "end_to_end_GBps": gathered * steps / wall / 1e9,
        "tier": {"gamma": gamma, "hit_rate_in": hit_in / max(look_in, 1), "hit_rate_mid": hit_mid / max(look_mid, 1),
                 "pcie_bytes_per_step": pcie / steps, "pcie_GBps": pcie / wall / 1e9},
        "kernels_us": {kname: v[0] / v[1] * 1e3 for kname, v in prof.items() if v[1]},
        "roofline": {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                     "traffic": None, "kernel": "gemv_kernel (up/gate + SwiGLU), rows from HBM slots or host memory",
                     "algorithmic_bytes_per_launch": ug_bytes, "avg_launch_us": ug_ms / ug_n * 1e3, "launches": ug_n},
    }
    print(json.dumps(out))


PAPER_TABLE2_PHI3_MEDIUM = {
    # context only: simulated Apple-A18 (DRAM 60 GB/s, Flash 1 GB/s), INT4 GPTQ, LFU cache,
    # model 7.4 GB with 4.0 GB of DRAM (Table 2, Phi-3-Medium column)
    "dense": 0.29, "dip_at_+0.2ppl": 0.43, "dip_ca_at_+0.2ppl": 0.45,
    "dip_at_+0.5ppl": 0.50, "dip_ca_at_+0.5ppl": 0.56,
}


def build_layers(D, cfg, L, workers=6):
    """Weights of L layers on the device (generated on host threads: numpy releases the GIL in
    its generators), layer 0 also kept on the host for the oracle sample."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from workloads import layer_weights

    d, f = cfg.d_model, cfg.d_ff
    if cfg.dtype == "int4":
        mk = lambda t: D.Weight(torch.from_numpy(t[0]).cuda(), torch.from_numpy(t[1]).cuda())
    else:
        mk = lambda arr: D.Weight(torch.from_numpy(arr.view(np.int16)).cuda())
    mlps, host0 = [], None
    with ThreadPoolExecutor(max_workers=workers) as pool:
        pending = []
        for l in range(L):
            pending.append(pool.submit(layer_weights, d, f, cfg.seed, l, cfg.dtype))
            # bounded look-ahead: a layer in fp32 on the host is over a gigabyte
            while pending and (len(pending) >= workers or l == L - 1):
                w = pending.pop(0).result()
                if host0 is None:
                    host0 = w
                mlps.append(D.Mlp(mk(w["ug"]), mk(w["d"])))
                del w
    return mlps, host0


def timed_repeats(one_block, blocks, repeats, min_repeat_ms):
    """Time `repeats` repeats of `blocks` blocks each, synchronised on both sides.  A repeat that
    comes out shorter than the minimum (the pilot block ran slower than the steady state) has its
    block count raised and the whole set is measured again, so every reported repeat lasts at
    least `min_repeat_ms`.  Returns (blocks, [seconds per repeat])."""
    import torch
    for _ in range(4):
        times = []
        for _ in range(max(1, repeats)):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(blocks):
                one_block()
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
        short = min(times) * 1e3
        if short >= min_repeat_ms:
            break
        blocks = int(np.ceil(blocks * 1.15 * min_repeat_ms / max(short, 1e-3)))
    return blocks, times


def hit_rates(D, cins, cmids, before=None):
    """Hit rates from the cache states' own counters (dip_cache.meta) through the two-tier
    model's reader; `before` = an earlier reading to take the difference with."""
    from paper_2412_01380_amd.twotier import hit_rates_from_meta
    mi = [c.meta_host() for c in cins]
    mm = [c.meta_host() for c in cmids]
    tot = {"in": {"cum_hits": sum(m["cum_hits"] for m in mi), "cum_lookups": sum(m["cum_lookups"] for m in mi)},
           "mid": {"cum_hits": sum(m["cum_hits"] for m in mm), "cum_lookups": sum(m["cum_lookups"] for m in mm)}}
    if before is None:
        return tot, hit_rates_from_meta(tot["in"], tot["mid"])
    diff = {p: {k: tot[p][k] - before[p][k] for k in tot[p]} for p in tot}
    return tot, hit_rates_from_meta(diff["in"], diff["mid"])


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X); --gpus must be 1. "
              "The path shards by layer or by output slice as the design notes describe, "
              "but no multi-GPU figure is produced.", file=sys.stderr)
        sys.exit(2)

    import ctypes as C
    import statistics
    import numpy as np
    import torch

    import paper_2412_01380_amd as D
    from paper_2412_01380_amd import twotier
    from workloads import CONFIGS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if a.tune:
        D.dip_tune_gemv(*[int(v) for v in a.tune.split(",")])
    if a.no_fusion:
        D.dip_set_fusion(False)
    if a.scheme != "dip":
        return bench_scheme(a)
    if a.tiered:
        return bench_tiered(a)
    torch.cuda.set_device(0)
    cfg = CONFIGS[a.config]
    r = a.ratio if a.ratio is not None else {2: 0.5, 3: 0.3, 4: 0.3, 5: 0.3}[a.config]
    frac = a.cache_frac if a.cache_frac is not None else {2: None, 3: 0.5, 4: 0.5, 5: 0.5}[a.config]
    gamma = a.gamma if a.gamma is not None else cfg.gamma
    policy = {"lru": D.DIP_LRU, "lfu": D.DIP_LFU}[a.policy]
    d, f = cfg.d_model, cfg.d_ff
    k_in, k_mid = cfg.k_in(r), cfg.k_mid(r)
    # config 2 is one layer shape: rotate over distinct weight copies so that the 256 MB
    # last-level cache cannot serve the reads; configs 3-5 are real stacks.
    L = a.layers if a.layers is not None else {2: 8}.get(a.config, cfg.n_layers)
    B = a.batch
    if B > 1:
        assert a.config == 5 and B <= 8, "--batch applies to config 5 (1..8 rows)"
    n_tok = min(cfg.n_tokens, a.tokens)

    t_setup = time.perf_counter()
    mlps, host0 = build_layers(D, cfg, L)
    # inputs: [token][layer][d]; every layer has its own stream (layers are not chained)
    X = np.stack([cfg.tokens(layer=l, n_tokens=n_tok) for l in range(L)], axis=1)
    Xd = torch.from_numpy(X).cuda()
    Yd = torch.empty(L, d, dtype=torch.float32, device="cuda")
    use_cache = frac is not None
    C_in = C_mid = None

    def fresh_caches(pol):
        ci = [D.Cache(d, C_in, pol) for _ in range(L)]
        cm = [D.Cache(f, C_mid, pol) for _ in range(L)]
        for c in ci + cm:
            D.dip_cache_init(c)
        return ci, cm

    cins = cmids = None
    if use_cache:
        C_in, C_mid = int(np.floor(frac * d + 0.5)), int(np.floor(frac * f + 0.5))
        cins, cmids = fresh_caches(policy)

    class Runner:
        """Issues layer-steps token-major: step s is layer s % L of token s // L.  A run of n
        steps is the tail of the current token, whole tokens, and the head of the next one,
        each a single call of the stack entry point over that range of layers."""

        def __init__(self, cins, cmids, gamma):
            self.cins, self.cmids, self.gamma = cins, cmids, gamma
            self.pos = 0
            self.ranges = {}
            full = D.MlpStack(mlps, cins, cmids)
            self.ws = torch.empty(D.dip_swiglu_mlp_forward_stack_workspace_bytes(full, k_in, k_mid),
                                  dtype=torch.uint8, device="cuda")

        def stack(self, l0, l1):
            if (l0, l1) not in self.ranges:
                m = l1 - l0
                self.ranges[(l0, l1)] = (
                    D.MlpStack(mlps[l0:l1], self.cins[l0:l1] if self.cins else None,
                               self.cmids[l0:l1] if self.cmids else None),
                    (C.c_int32 * m)(*([k_in] * m)), (C.c_int32 * m)(*([k_mid] * m)))
            return self.ranges[(l0, l1)]

        def run(self, n):
            while n > 0:
                t, l = divmod(self.pos, L)
                m = min(n, L - l)
                st, ki, km = self.stack(l, l + m)
                D.dip_swiglu_mlp_forward_stack(st, Xd[t % n_tok, l:], d, ki, km, self.gamma, Yd[l:], d, self.ws)
                self.pos += m
                n -= m

    if B > 1:
        return bench_batched(a, D, cfg, mlps, host0, X, Xd, cins, cmids, L, B, r, frac, gamma, k_in, k_mid, t_setup)

    run = Runner(cins, cmids, gamma)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup

    K, W = max(1, a.steps), max(0, a.warmup)
    # prepare every layer range a block of K steps can need, so that no descriptor is built inside a timed region
    run.run(W)
    torch.cuda.synchronize()
    pos0 = run.pos
    seen = set()
    for blk in range(L + 1):
        s0 = (pos0 + blk * K) % L
        if s0 in seen:
            break
        seen.add(s0)
        n, l = K, s0
        while n > 0:
            m = min(n, L - l)
            run.stack(l, l + m)
            n -= m
            l = 0
    # pilot block (untimed for the result): how many blocks make a repeat of >= 20 ms
    t0 = time.perf_counter()
    run.run(K)
    torch.cuda.synchronize()
    pilot = time.perf_counter() - t0
    blocks = max(1, int(np.ceil(1.25 * a.min_repeat_ms * 1e-3 / max(pilot, 1e-6))))
    hr_before = hit_rates(D, cins, cmids)[0] if use_cache else None
    one_block = lambda: run.run(K)            # exactly K layer-steps
    launch_mode = "launches issued from the host through dip_swiglu_mlp_forward_stack"
    if a.graph:
        # The launches of one block are captured once into a HIP graph (the library only
        # launches kernels on the given stream: no allocation, no memset, no host
        # synchronisation) and the block is replayed: same kernels, same arguments, same
        # tokens.  Cache state lives in device memory and keeps evolving from replay to replay.
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run.run(K)
        graph.replay()                        # one untimed replay
        torch.cuda.synchronize()
        one_block = graph.replay
        launch_mode = f"HIP graph of one block of {K} steps, replayed"
    blocks, times = timed_repeats(one_block, blocks, a.repeats, a.min_repeat_ms)
    wall = statistics.median(times)
    ms_per_step = wall / (blocks * K) * 1e3
    steps_per_s = 1e3 / ms_per_step

    gathered = cfg.gathered_bytes(r)
    bytes_of = (lambda e: e // 2 + (e // 128) * 2) if cfg.dtype == "int4" else (lambda e: e * 2)
    ug_bytes = bytes_of(2 * k_in * f)
    dn_bytes = bytes_of(k_mid * d)
    fused_ug = D.dip_fused_launch_shape(mlps[0].w_ug, k_in, bundled=True)
    fused_dn = D.dip_fused_launch_shape(mlps[0].w_d, k_mid, bundled=False)
    launches = (1 if fused_ug else 2) + (1 if fused_dn else 2)
    out = {
        "metric": "DIP MLP decode tokens/s at batch 1 + achieved HBM GB/s vs peak on gathered bytes",
        "value": steps_per_s,
        "unit": "layer-tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": f"BASELINE configs[{a.config - 1}]: {cfg.name}, d_model={d}, d_ff={f}, "
                        f"{cfg.dtype} weights, batch 1, keep ratio {r} (k_in={k_in}, k_mid={k_mid}), "
                        + (f"DIP-CA {a.policy.upper()} cache frac {frac} (C_in={C_in}, C_mid={C_mid}), gamma {gamma}"
                           if use_cache else "DIP only")
                        + f", {L} " + ("distinct weight copies visited round-robin" if a.config == 2
                                        else "layers per token, walked token-major"),
            "inputs": cfg.inputs, "weights_dtype": cfg.dtype,
            "weight_bytes_resident": int(L * bytes_of(3 * d * f)),
            "gathered_bytes_per_step": gathered,
            "step": f"one token through one MLP layer ({launches} kernel launches"
                    + (", cache updates of a token's layers batched into one more" if use_cache else "") + ")",
            "batch": 1,
            "launch": launch_mode,
        },
        "timing": {"repeats": len(times), "blocks_per_repeat": blocks, "steps_per_block": K,
                   "repeat_ms": [t * 1e3 for t in times], "statistic": "median of repeats",
                   "pilot_block_ms": pilot * 1e3},
        "tokens_per_s": steps_per_s / L if a.config != 2 else None,
        "layers_per_token": L if a.config != 2 else None,
        "end_to_end_GBps": gathered * steps_per_s / 1e9,
        "end_to_end_frac_of_peak": gathered * steps_per_s / 1e9 / HBM_PEAK_GBS,
        "setup_s": t_setup,
    }
    if use_cache:
        _, (hi, hm) = hit_rates(D, cins, cmids, hr_before)
        out["cache_hit_rate"] = {"in": hi, "mid": hm, "policy": a.policy, "gamma": gamma,
                                 "window": "the timed repeats"}

    if a.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")     # 1 GiB read
        dst = torch.empty_like(src)                                        # 1 GiB written
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["calibration_copy_bytes"] = {"read": int(src.numel() * 4), "written": int(dst.numel() * 4)}
        del src, dst

    # ---- per-kernel durations from HIP events bound to the dispatches ---------------------
    ceiling = None
    if not a.no_kernel_events:
        n_prof = min(max(K, 4 * L), 4096)
        D.dip_profile_enable(5 * n_prof + 64)
        run.run(n_prof)
        torch.cuda.synchronize()
        names = ("select_in", "gemv_upgate", "select_mid", "gemv_down")
        prof = {k: D.dip_profile_read(i) for i, k in enumerate(names)}
        prof["cache_updates"] = D.dip_profile_read(7)
        D.dip_profile_disable()
        out["kernels_us"] = {k: (v[0] / v[1] * 1e3 if v[1] else None) for k, v in prof.items()}
        out["launches_per_step"] = sum(v[1] for v in prof.values()) / n_prof
        # a plain streaming read of 4 GiB in the same run: the ceiling a load-only kernel reaches here
        buf = torch.zeros(1 << 30, dtype=torch.int32, device="cuda")
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        D.dip_stream_read(buf, sink)
        torch.cuda.synchronize()
        D.dip_profile_enable(16)
        for _ in range(5):
            D.dip_stream_read(buf, sink)
        torch.cuda.synchronize()
        ms, n = D.dip_profile_read(8)
        D.dip_profile_disable()
        ceiling = buf.numel() * 4 / (ms / n * 1e-3) / 1e9
        del buf
        shape_ug = fused_ug or D.dip_gemv_launch_shape(mlps[0].w_ug, k_in, bundled=True)
        shape_dn = fused_dn or D.dip_gemv_launch_shape(mlps[0].w_d, k_mid, bundled=False)
        out["launch_shapes"] = {"gemv_upgate": list(shape_ug), "gemv_down": list(shape_dn),
                                "fields": "lanes_per_row, waves, ksplit, unroll",
                                "selection_inside_the_product": [bool(fused_ug), bool(fused_dn)]}
        ug_ms, ug_n = prof["gemv_upgate"]
        dn_ms, dn_n = prof["gemv_down"]
        if ug_n:
            ach = ug_bytes / (ug_ms / ug_n * 1e-3) / 1e9
            out["roofline"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                               "frac": ach / HBM_PEAK_GBS,
                               "traffic": measured_traffic(cfg.name, r, shape_ug),
                               "kernel": ("fused_kernel (scores + top-K + gathered up/gate + SwiGLU in one launch)"
                                          if fused_ug else "gemv_kernel (up/gate + SwiGLU)"),
                               "algorithmic_bytes_per_launch": ug_bytes,
                               "avg_launch_us": ug_ms / ug_n * 1e3, "launches": ug_n,
                               "ceiling_GBps": ceiling, "frac_of_ceiling": ach / ceiling}
        if dn_n:
            ach = dn_bytes / (dn_ms / dn_n * 1e-3) / 1e9
            out["roofline_down"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": ach / HBM_PEAK_GBS,
                                    "kernel": ("fused_kernel (scores + top-K + gathered down in one launch)"
                                               if fused_dn else "gemv_kernel (down)"),
                                    "algorithmic_bytes_per_launch": dn_bytes,
                                    "avg_launch_us": dn_ms / dn_n * 1e3, "launches": dn_n,
                                    "ceiling_GBps": ceiling, "frac_of_ceiling": ach / ceiling}

    # ---- eviction policies and the penalty, on fresh caches (Sec. 6.4), and what the measured hit
    #      rates mean on the paper's simulated phone (Sec. 6.1, App. A) --------------------------
    if use_cache and not a.no_side_runs:
        side = {}
        n_side, n_skip = a.side_tokens, a.side_tokens // 3
        # int4 column sizes of this shape: the paper's throughput runs are INT4
        col_in, col_mid = 2 * (f // 2 + (f // 128) * 2), d // 2 + (d // 128) * 2
        mlp_bytes = L * (d * col_in + f * col_mid)
        static_bytes = max(0.0, 7.4e9 - mlp_bytes) if a.config in (4, 5) else 0.0
        for pol_name in ("lru", "lfu"):
            for g in (1.0, gamma):
                ci, cm = fresh_caches({"lru": D.DIP_LRU, "lfu": D.DIP_LFU}[pol_name])
                rr = Runner(ci, cm, g)
                rr.run(n_skip * L)
                torch.cuda.synchronize()
                before = hit_rates(D, ci, cm)[0]
                rr.run((n_side - n_skip) * L)
                torch.cuda.synchronize()
                _, (hi, hm) = hit_rates(D, ci, cm, before)
                sim = twotier.sparse_tokens_per_second(static_bytes, L, col_in, col_mid, k_in, k_mid, hi, hm)
                side[f"{pol_name}_gamma{g:g}"] = {"hit_rate_in": hi, "hit_rate_mid": hm,
                                                  "simulated_mobile_tokens_per_s": sim}
                del rr, ci, cm
        out["eviction_policies"] = {
            "runs": side,
            "procedure": f"fresh caches, {n_side} tokens through all {L} layers, hit rates over the last "
                         f"{n_side - n_skip}; gamma 1 is plain DIP (keys |x|)",
            "mobile_model": "bytes missed / 1 GB/s Flash against bytes used / 60 GB/s DRAM (Sec. 6.1), INT4 column "
                            f"sizes of this shape, {static_bytes / 1e9:.2f} GB of never-pruned weights pinned in DRAM",
            "paper_table2_phi3_medium_context": PAPER_TABLE2_PHI3_MEDIUM,
        }

    # ---- the oracle on the host cores, bounded sample --------------------------------------
    if not a.no_cpu_baseline:
        from oracle import dip_oracle as O
        nt = a.cpu_sample_tokens
        oc_in = O.CacheState(n=d, capacity=C_in, policy=a.policy) if use_cache else None
        oc_mid = O.CacheState(n=f, capacity=C_mid, policy=a.policy) if use_cache else None
        c0, w0t = time.process_time(), time.perf_counter()
        for t in range(nt):
            O.mlp_forward(host0["ug"], host0["d"], X[t % n_tok, 0], k_in, k_mid, oc_in, oc_mid, gamma)
        wall_o = time.perf_counter() - w0t
        cpu_o = time.process_time() - c0
        out["cpu_baseline"] = {
            "value": nt / wall_o, "unit": out["unit"], "cores": max(1, int(round(cpu_o / wall_o))),
            "kind": "oracle",
            "sample": f"{nt} tokens through layer 0 of the same workload "
                      f"({wall_o:.1f} s wall, {cpu_o:.1f} s CPU; host has {len(os.sched_getaffinity(0))} usable cores)"}
    print(json.dumps(out))


def bench_batched(a, D, cfg, mlps, host0, X, Xd, cins, cmids, L, B, r, frac, gamma, k_in, k_mid, t_setup):
    """Config 5 at batch B > 1: B rows per step through one layer, columns read once per step
    if any row selected them.  Bytes are the MEASURED union sizes times the column sizes."""
    import ctypes as C
    import numpy as np
    import statistics
    import torch

    d, f = cfg.d_model, cfg.d_ff
    n_tok = Xd.shape[0]
    use_cache = cins is not None
    # row b of layer l at step t is its own stream: shifted copies of the layer's stream
    Xb = torch.stack([Xd[(torch.arange(n_tok) + 37 * b) % n_tok] for b in range(B)], dim=2).contiguous()
    Yb = torch.empty(L, B, d, dtype=torch.float32, device="cuda")
    ws1 = torch.empty(D.dip_swiglu_mlp_forward_batched_workspace_bytes(mlps[0], B, k_in, k_mid),
                      dtype=torch.uint8, device="cuda")
    wd, wf = (d + 31) // 32, (f + 31) // 32
    m_in = torch.zeros(B, wd, dtype=torch.int32, device="cuda")
    m_mid = torch.zeros(B, wf, dtype=torch.int32, device="cuda")
    pos = [0]
    ranges = {}
    full = D.MlpStack(mlps, cins, cmids)
    ws = torch.empty(D.dip_swiglu_mlp_forward_batched_stack_workspace_bytes(full, B, k_in, k_mid),
                     dtype=torch.uint8, device="cuda")

    def stack(l0, l1):
        if (l0, l1) not in ranges:
            m = l1 - l0
            ranges[(l0, l1)] = (D.MlpStack(mlps[l0:l1], cins[l0:l1] if use_cache else None,
                                           cmids[l0:l1] if use_cache else None),
                                (C.c_int32 * m)(*([k_in] * m)), (C.c_int32 * m)(*([k_mid] * m)))
        return ranges[(l0, l1)]

    def run(n, masks=False):
        """n layer-steps, token-major; each range of layers of one token is one call of the batched
        stack entry point (with `masks`: one layer per call, so that its row masks can be read)."""
        while n > 0:
            t, l = divmod(pos[0], L)
            if masks:
                D.dip_swiglu_mlp_forward_batched(mlps[l], Xb[t % n_tok, l], B, k_in, k_mid,
                                                 cins[l] if use_cache else None, cmids[l] if use_cache else None,
                                                 gamma, Yb[l], m_in, None, m_mid, ws1)
                m = 1
            else:
                m = min(n, L - l)
                st, ki, km = stack(l, l + m)
                D.dip_swiglu_mlp_forward_batched_stack(st, Xb[t % n_tok, l:], B * d, B, ki, km, gamma, Yb[l:], B * d, ws)
            pos[0] += m
            n -= m

    K, W = max(1, a.steps), max(0, a.warmup)
    run(W)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t_setup
    t0 = time.perf_counter()
    run(K)
    torch.cuda.synchronize()
    pilot = time.perf_counter() - t0
    blocks = max(1, int(np.ceil(1.25 * a.min_repeat_ms * 1e-3 / max(pilot, 1e-6))))
    blocks, times = timed_repeats(lambda: run(K), blocks, a.repeats, a.min_repeat_ms)
    wall = statistics.median(times)
    ms_per_step = wall / (blocks * K) * 1e3

    # measured union sizes: |U_in|, |U_mid| averaged over sample steps
    def popcount_union(m):
        u = m[0]
        for b in range(1, B):
            u = u | m[b]
        return int(np.unpackbits(u.cpu().numpy().view(np.uint8)).sum())
    ns, u_in, u_mid = 32, 0, 0
    for _ in range(ns):
        run(1, masks=True)
        torch.cuda.synchronize()
        u_in += popcount_union(m_in)
        u_mid += popcount_union(m_mid)
    u_in, u_mid = u_in / ns, u_mid / ns
    col_in, col_mid = 2 * (f // 2 + (f // 128) * 2), d // 2 + (d // 128) * 2
    ug_bytes, dn_bytes = u_in * col_in, u_mid * col_mid
    gathered = ug_bytes + dn_bytes

    n_prof = min(K, 512)
    D.dip_profile_enable(12 * n_prof + 64)
    run(n_prof)
    torch.cuda.synchronize()
    names = ("select_in", "gemv_upgate", "select_mid", "gemv_down")
    prof = {k: D.dip_profile_read(i) for i, k in enumerate(names)}
    D.dip_profile_disable()
    ug_ms, ug_n = prof["gemv_upgate"]
    dn_ms, dn_n = prof["gemv_down"]
    ach = ug_bytes / (ug_ms / ug_n * 1e-3) / 1e9

    # Which roofline binds a batched product: HBM on the bytes of the union, or the plain vector
    # ALU on the arithmetic every stored code costs -- B multiply-adds (2 B flops) plus about 3
    # operations to unpack it -- against 157.3 TFLOP/s (256 compute units x 4 x 64-lane fp32 FMA
    # per 4 cycles x 2.4 GHz).  From 3 rows on the multiply-adds of int4 weights run on the matrix
    # cores, the unpacking stays on the vector ALU; the vector-ALU model is quoted for every B.
    def two_bounds(n_cols, codes_per_col, nbytes, us):
        ops = n_cols * codes_per_col * (2 * B + 3)
        t_hbm, t_alu = nbytes / (HBM_PEAK_GBS * 1e9), ops / (VALU_PEAK_TFLOPS * 1e12)
        hbm = {"achieved_GBps": nbytes / (us * 1e-6) / 1e9, "peak_GBps": HBM_PEAK_GBS,
               "frac": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, "model_us": t_hbm * 1e6}
        alu = {"achieved_TFLOPs": ops / (us * 1e-6) / 1e12, "peak_TFLOPs": VALU_PEAK_TFLOPS,
               "frac": ops / (us * 1e-6) / 1e12 / VALU_PEAK_TFLOPS, "model_us": t_alu * 1e6, "ops_per_launch": ops}
        return ("alu" if t_alu > t_hbm else "hbm"), hbm, alu
    ug_us, dn_us = ug_ms / ug_n * 1e3, dn_ms / dn_n * 1e3
    ug_bound, ug_hbm, ug_alu = two_bounds(u_in, 2 * f, ug_bytes, ug_us)
    dn_bound, dn_hbm, dn_alu = two_bounds(u_mid, d, dn_bytes, dn_us)

    def roof(bound, hbm, alu, **extra):
        o = ({"bound": "alu", "achieved": alu["achieved_TFLOPs"], "peak": VALU_PEAK_TFLOPS, "unit": "TFLOP/s",
              "frac": alu["frac"]} if bound == "alu" else
             {"bound": "hbm", "achieved": hbm["achieved_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
              "frac": hbm["frac"]})
        o.update({"traffic": None, "hbm": hbm, "alu": alu,
                  "binds": f"{bound} (model: {hbm['model_us']:.1f} us of HBM, {alu['model_us']:.1f} us of vector ALU)"})
        o.update(extra)
        return o
    out = {
        "metric": "DIP MLP decode tokens/s at batch 1 + achieved HBM GB/s vs peak on gathered bytes",
        "value": B * 1e3 / ms_per_step, "unit": "row-layers/s (rows x layer-steps per second)",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": f"BASELINE configs[{a.config - 1}]: {cfg.name}, d_model={d}, d_ff={f}, {cfg.dtype} weights, "
                        f"batch {B} (per-row top-K masks, unioned column reads), keep ratio {r} "
                        f"(k_in={k_in}, k_mid={k_mid}), "
                        + (f"DIP-CA {a.policy.upper()} cache frac {frac}, gamma {gamma}" if use_cache else "DIP only")
                        + f", {L} layers per token, walked token-major",
            "inputs": cfg.inputs, "weights_dtype": cfg.dtype, "batch": B,
            "measured_union_columns": {"in": u_in, "mid": u_mid, "of": [d, f], "sample_steps": ns},
            "gathered_bytes_per_step": gathered,
            "step": f"{B} rows through one MLP layer (dip_swiglu_mlp_forward_batched_stack over the layers of a token)",
        },
        "timing": {"repeats": len(times), "blocks_per_repeat": blocks, "steps_per_block": K,
                   "repeat_ms": [t * 1e3 for t in times], "statistic": "median of repeats"},
        "tokens_per_s": B * 1e3 / ms_per_step / L,
        "end_to_end_GBps": gathered / (ms_per_step * 1e-3) / 1e9,
        "setup_s": t_setup,
        "kernels_us": {k: (v[0] / v[1] * 1e3 if v[1] else None) for k, v in prof.items()},
        "roofline": roof(ug_bound, ug_hbm, ug_alu,
                         kernel="batched gathered product (up/gate), bytes and codes of the measured union",
                         algorithmic_bytes_per_launch=ug_bytes, avg_launch_us=ug_us, launches=ug_n),
        "roofline_down": roof(dn_bound, dn_hbm, dn_alu,
                              kernel="batched gathered product (down), bytes and codes of the measured union",
                              algorithmic_bytes_per_launch=dn_bytes, avg_launch_us=dn_us, launches=dn_n),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
