#!/usr/bin/env python3
"""Benchmark of the clustered-head decode attention path on one MI355X.

A step = one decode token for every batch row through the attention of ALL layers of the configuration
(scores of each cluster over the compact K cache, stable softmax, shared probabilities applied to every head's
own V cache).  Caches, queries and cluster maps are resident in HBM before the timed region; membership comes
from the library's own feature + k-means + compaction kernels (or from the drawn partition for the configurations
that prescribe one).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cfg2]
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--context", type=int, default=0, help="override the number of cached tokens (cfg4: 640 or 2048)")
    ap.add_argument("--mode", default="decode", choices=["decode", "prefill", "shared-v", "project", "e2e", "q8"],
                    help="decode (default, the headline metric), the clustered prefill attention, the decode "
                         "ablation that prunes values as well, or the query/key projections of the representatives")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-phase-timing", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="default run only: skip the records of the other four configurations")
    ap.add_argument("--settle", type=float, default=3.0,
                    help="default run only: idle seconds before each of the other configurations, so that each is "
                         "timed from the clock state a run of its own would start in (back to back they read about "
                         "4 %% lower: the card lowers its clocks after some seconds of sustained load)")
    return ap.parse_args()


class Layer:
    __slots__ = ("k", "q", "kfull", "kc", "v", "h2c", "rep", "out")


def build_layers(cfg, W, C, torch, keep_full_k):
    """Allocate and fill every layer's tensors on the device; run membership + compaction through the library."""
    dev = "cuda"
    B, H, d, T, T_cap = cfg.B, cfg.H, cfg.d, cfg.T, cfg.T_cap
    tdt = torch.float32 if cfg.dtype == W.F32 else torch.bfloat16
    layers = []
    t_member = 0.0
    for l in range(cfg.L):
        k = cfg.ks[l]
        L = Layer()
        L.k = k
        seed = cfg.seed * 100003 + l * 17
        groups = None
        if cfg.membership == "planted":
            groups = W.planted_partition(W.rng(cfg.seed, l, "planted"), B, H, k)
            kfull = W.device_centroid_plus_noise(groups, k, T_cap, d, cfg.dtype, seed + 1, dev)
            q5 = W.device_centroid_plus_noise(groups, k, W.N_TOK, d, cfg.dtype, seed + 3, dev)
            L.q = W.device_centroid_plus_noise(groups, k, 1, d, cfg.dtype, seed + 5, dev)[:, :, 0, :].contiguous()
        else:
            kfull = W.device_normal((B, H, T_cap, d), cfg.dtype, seed + 1, dev)
            q5 = W.device_normal((B, H, W.N_TOK, d), cfg.dtype, seed + 3, dev)
            L.q = W.device_normal((B, H, d), cfg.dtype, seed + 5, dev)
        L.v = W.device_normal((B, H, T_cap, d), cfg.dtype, seed + 7, dev)
        L.out = torch.empty((B, H, d), dtype=torch.float32, device=dev)

        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if cfg.membership in ("kmeans", "planted"):
            if cfg.membership == "planted":
                init = W.one_head_per_group(W.rng(cfg.seed, l, "init"), groups, k)
            else:
                init = W.distinct_heads(W.rng(cfg.seed, l, "init"), B, H, k)
            feat = C.chai_score_features(q5, kfull, W.N_TOK, cfg.scale)
            L.h2c, L.rep, _, _ = C.chai_assign_clusters(feat, W.host_to_torch(init, dev))
        else:
            g = W.rng(cfg.seed, l, "member")
            h2c, rep = (W.sized_membership(g, B, H, cfg.sizes) if cfg.membership == "skewed"
                        else W.random_membership(g, B, H, k))
            L.h2c, L.rep = W.host_to_torch(h2c, dev), W.host_to_torch(rep, dev)
        L.kc = torch.empty((B, k, T_cap, d), dtype=tdt, device=dev)
        C.chai_compact_kcache(kfull, L.rep, L.kc, T)
        torch.cuda.synchronize()
        t_member += time.perf_counter() - t0
        L.kfull = kfull if keep_full_k else None
        del kfull, q5
        layers.append(L)
    return layers, t_member


def timed_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return e0.elapsed_time(e1) / steps, wall


class HipEvents:
    """hipEvent_t handles from the HIP runtime that is already loaded in this process (torch's), so that the
    library can have the runtime stamp the begin and the end of a kernel into them."""

    def __init__(self):
        import ctypes
        paths = sorted({l.split()[-1] for l in open("/proc/self/maps") if "libamdhip64" in l})
        if not paths:
            raise RuntimeError("no HIP runtime loaded")
        self.ct = ctypes
        self.hip = ctypes.CDLL(paths[0])
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.made = []

    def create(self) -> int:
        ev = self.ct.c_void_p()
        rc = self.hip.hipEventCreate(self.ct.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed ({rc})")
        self.made.append(ev.value)
        return ev.value

    def elapsed_ms(self, a: int, b: int) -> float:
        ms = self.ct.c_float()
        rc = self.hip.hipEventElapsedTime(self.ct.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def close(self):
        for ev in self.made:
            self.hip.hipEventDestroy(ev)
        self.made = []


def phase_timing(layers, cfg, ws, C, torch, steps):
    """Average duration of the score kernel and of the value kernel per launch over `steps` more steps of the same
    workload.  Each launch carries a pair of HIP events that the runtime stamps with the kernel's own begin and end
    on the launch stream (so launch gaps are not counted, as in a profiler's kernel trace); a separate pass, so
    the events do not perturb the headline timing."""
    hev = HipEvents()
    recs = []
    for _ in range(steps):
        for li, L in enumerate(layers):
            e = [hev.create() for _ in range(4)]
            C.chai_decode_scores_timed(L.q, L.kc, L.rep, cfg.T, cfg.scale, ws, start_event=e[0], stop_event=e[1])
            C.chai_decode_values_timed(L.v, L.h2c, L.rep, cfg.T, L.out, ws, start_event=e[2], stop_event=e[3])
            recs.append((li, e))
    torch.cuda.synchronize()
    per_layer = {}
    for li, e in recs:
        s, v = per_layer.get(li, (0.0, 0.0))
        per_layer[li] = (s + hev.elapsed_ms(e[0], e[1]), v + hev.elapsed_ms(e[2], e[3]))
    hev.close()
    return {li: (s / steps, v / steps) for li, (s, v) in per_layer.items()}


def read_ceiling(layers, C, torch):
    """Rate of a bare streaming read (the library's probe kernel) over the resident value caches, one launch per
    layer, timed with events stamped at each kernel's begin and end: the practical ceiling of the HBM-bound
    kernels on this device."""
    hev = HipEvents()
    sink = torch.zeros((1,), dtype=torch.float32, device="cuda")
    recs = []
    for rep in range(3):
        for L in layers[:16]:
            e0, e1 = hev.create(), hev.create()
            C.chai_stream_read_probe(L.v, sink, start_event=e0, stop_event=e1)
            recs.append((rep, L.v.numel() * L.v.element_size(), e0, e1))
    torch.cuda.synchronize()
    rates = sorted(nb / (hev.elapsed_ms(e0, e1) * 1e-3) / 1e9 for rep, nb, e0, e1 in recs if rep > 0)
    hev.close()
    return rates[len(rates) // 2]


def mfma_ceiling(data, C, torch):
    """Rate of the matrix pipe alone (the library's probe kernel) on operands taken from the workload's own data,
    in TFLOP/s: what the bf16 MFMAs reach on this device with these values when nothing else is in the way."""
    hev = HipEvents()
    sink = torch.zeros((1,), dtype=torch.float32, device="cuda")
    recs = []
    for rep in range(4):
        e0, e1 = hev.create(), hev.create()
        fl = C.chai_mfma_rate_probe(data, 4000, sink, start_event=e0, stop_event=e1)
        recs.append((fl, e0, e1))
    torch.cuda.synchronize()
    rates = sorted(fl / (hev.elapsed_ms(e0, e1) * 1e-3) / 1e12 for fl, e0, e1 in recs[1:])
    hev.close()
    return rates[len(rates) // 2]


def read_traffic(cfg_name, kernel="value_kernel"):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{cfg_name}_hbm_traffic.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def cpu_baseline(cfg, layers, W, torch, budget_s=60.0):
    """The CPU oracle, as it stands, timed on the same workload: every batch row of every layer (a full step), as
    long as the sweep stays inside `budget_s` seconds of oracle time; if a configuration is too large for that,
    the layers done so far are scaled to a full step by bytes streamed and the record says so.  The oracle reads
    the FULL key cache and indexes the representative itself, so the comparison of its outputs with the GPU's
    (parity re-check on the timed tensors) also covers the compaction."""
    import numpy as np
    from oracle import chai_oracle as O
    spent, worst, done_layers, done_rows = 0.0, 0.0, 0, 0
    for li, L in enumerate(layers):
        if L.kfull is None:
            raise RuntimeError("cpu_baseline needs the full key caches (run without --no-dense)")
        h2c, rep = L.h2c.cpu().numpy(), L.rep.cpu().numpy()
        q, kf, v = W.torch_to_host_bits(L.q), W.torch_to_host_bits(L.kfull), W.torch_to_host_bits(L.v)
        t0 = time.perf_counter()
        ref = O.clustered_decode(q, kf, v, h2c, rep, cfg.T, cfg.scale)
        spent += time.perf_counter() - t0
        got = L.out.cpu().numpy().astype(np.float64)
        worst = max(worst, float((np.abs(got - ref).max(-1) / np.abs(ref).max(-1)).max()))
        done_layers += 1
        done_rows += L.k + cfg.H
        del kf, v
        if spent > budget_s:
            break
    all_rows = sum(L.k + cfg.H for L in layers)
    step_s = spent * all_rows / done_rows
    full = done_layers == len(layers)
    sample = (f"the whole step: all {cfg.B} batch rows of all {cfg.L} layers ({spent:.2f} s of oracle time, nothing "
              f"extrapolated)" if full else
              f"all {cfg.B} batch rows of the first {done_layers} of {cfg.L} layers ({spent:.1f} s of oracle time), "
              f"scaled to all layers by rows streamed (extrapolated)")
    return {"value": cfg.B / step_s, "unit": "tokens/s", "cores": O.num_threads(), "kind": "oracle", "sample": sample,
            "ms_per_step": step_s * 1e3, "parity_worst_normwise_err": worst,
            "parity_note": "oracle fed the full key cache, not the compact one"}


def sampled_parity(cfg, layers, W, torch, n_layers=2, n_heads=6):
    """Oracle on a few sampled (batch row, head) pairs of a few layers, from the FULL key cache (so a compaction
    error shows): worst normwise error relative to the row's largest element."""
    import numpy as np
    from oracle import chai_oracle as O
    g = np.random.default_rng(cfg.seed)
    idx = sorted(set(int(round(i * (len(layers) - 1) / max(n_layers - 1, 1))) for i in range(n_layers)))
    worst = 0.0
    for li in idx:
        L = layers[li]
        h2c, rep = L.h2c.cpu().numpy(), L.rep.cpu().numpy()
        for _ in range(n_heads):
            b, h = int(g.integers(cfg.B)), int(g.integers(cfg.H))
            r = int(rep[b, h2c[b, h]])
            q = np.stack([W.torch_to_host_bits(L.q[b, r]), W.torch_to_host_bits(L.q[b, r]) * 0])[None]
            kr = W.torch_to_host_bits(L.kfull[b, r] if L.kfull is not None else L.kc[b, h2c[b, h]])
            vh = W.torch_to_host_bits(L.v[b, h])
            ref = O.clustered_decode(q, np.stack([kr, kr * 0])[None], np.stack([vh * 0, vh])[None],
                                     np.zeros((1, 2), np.int32), np.zeros((1, 1), np.int32), cfg.T, cfg.scale)[0, 1]
            got = L.out[b, h].cpu().numpy().astype(np.float64)
            worst = max(worst, float(np.abs(got - ref).max() / np.abs(ref).max()))
    return {"worst_normwise_err": worst, "layers": idx, "heads_per_layer": n_heads,
            "key_source": "full key cache" if layers[0].kfull is not None else "compact key cache"}


def prefill_main(args, cfg, torch, C, W):
    """Clustered prefill attention (the block of prompt positions after the membership decision) of all layers of
    the configuration: one step = B prompts of cfg.T tokens through every layer's attention.  Four layers' tensors
    are resident and visited in turn (their working set is far beyond the caches)."""
    import numpy as np
    B, H, d, T = cfg.B, cfg.H, cfg.d, cfg.T
    q_start = W.N_TOK
    Tq = T - q_start
    n_res = min(cfg.L, 4)
    layers = []
    for l in range(n_res):
        k = cfg.ks[(l * cfg.L) // n_res if cfg.L > n_res else l]
        seed = cfg.seed * 7919 + l
        L = Layer()
        L.k = k
        g = W.rng(cfg.seed, l, "member")
        if cfg.membership == "skewed":
            h2c, rep = W.sized_membership(g, B, H, cfg.sizes)
        else:
            h2c, rep = W.random_membership(g, B, H, k)
        L.h2c, L.rep = W.host_to_torch(h2c), W.host_to_torch(rep)
        L.q = W.device_normal((B, H, Tq, d), cfg.dtype, seed + 1)
        L.kfull = W.device_normal((B, H, T, d), cfg.dtype, seed + 2)
        L.v = W.device_normal((B, H, T, d), cfg.dtype, seed + 3)
        L.kc = torch.empty((B, k, T, d), dtype=torch.bfloat16, device="cuda")
        C.chai_compact_kcache(L.kfull, L.rep, L.kc, T)
        L.out = torch.empty((B, H, Tq, d), dtype=torch.float32, device="cuda")
        layers.append(L)
    ws = torch.empty((C.chai_prefill_workspace_bytes(B, H, H, T),), dtype=torch.uint8, device="cuda")
    ks_all = [layers[(l * n_res) // cfg.L].k for l in range(cfg.L)]

    def clustered_step():
        for l in range(cfg.L):
            L = layers[(l * n_res) // cfg.L]
            C.chai_prefill_attention(L.q, L.kc, L.v, L.h2c, L.rep, q_start, cfg.scale, L.out, ws)

    def dense_step():
        for l in range(cfg.L):
            L = layers[(l * n_res) // cfg.L]
            C.chai_dense_prefill_attention(L.q, L.kfull, L.v, q_start, cfg.scale, L.out, ws)

    steps, warmup = max(args.steps // 4, 2), max(args.warmup // 2, 1)
    dense_ms = None
    if not args.no_dense:
        dense_ms, _ = timed_steps(dense_step, max(steps // 2, 1), warmup, torch)
    ms, wall_ms = timed_steps(clustered_step, steps, warmup, torch)
    pairs = sum(q_start + i + 1 for i in range(Tq))                      # (query, key) pairs under the causal mask
    layer_flops = {k: 2 * d * pairs * B * (k + H) for k in set(ks_all)}  # one score + one value product per pair
    flops = sum(layer_flops[k] for k in ks_all)
    dense_flops = 2 * d * pairs * B * 2 * H * cfg.L
    # the main kernel alone: events stamped by the runtime at its begin and end, in a pass of its own
    kern = {}
    if not args.no_phase_timing:
        hev = HipEvents()
        recs = []
        for _ in range(max(steps // 2, 1)):
            for l in range(cfg.L):
                L = layers[(l * n_res) // cfg.L]
                e0, e1 = hev.create(), hev.create()
                C.chai_prefill_attention_timed(L.q, L.kc, L.v, L.h2c, L.rep, q_start, cfg.scale, L.out, ws,
                                               start_event=e0, stop_event=e1)
                recs.append((L.k, e0, e1))
        torch.cuda.synchronize()
        for k, e0, e1 in recs:
            kern.setdefault(k, []).append(hev.elapsed_ms(e0, e1))
        hev.close()
    if kern:
        # dominant launch shape = the cluster count most layers use
        k_dom = max(set(ks_all), key=ks_all.count)
        kms = sum(kern[k_dom]) / len(kern[k_dom])
        ach = layer_flops[k_dom] / (kms * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": f"prefill_kernel, layers with {k_dom} clusters", "achieved": ach,
                "peak": 2500.0, "unit": "TFLOP/s", "frac": ach / 2500.0,
                "traffic": read_traffic(cfg.name, "prefill_kernel") if T == W.CONFIGS[cfg.name].T else None,
                "avg_launch_ms": kms, "flops_per_launch": layer_flops[k_dom],
                "kernel_ms_by_clusters": {str(k): sum(v) / len(v) for k, v in sorted(kern.items())}}
        ceil_tf = mfma_ceiling(layers[-1].q, C, torch)
        roof["mfma_ceiling"] = {"TFLOPs": ceil_tf, "frac_of_peak": ceil_tf / 2500.0, "kernel_frac_of_ceiling": ach / ceil_tf,
                                "how": "matrix pipe alone on the workload's query data (chai_mfma_rate_probe)"}
    else:
        ach = flops / (ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": "whole call (V^T pre-pass, work list, prefill_kernel)", "achieved": ach,
                "peak": 2500.0, "unit": "TFLOP/s", "frac": ach / 2500.0, "traffic": None}
    result = {
        "metric": "clustered prefill attention prompt tokens/s (attention of all layers)",
        "value": B * Tq / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name} prefill: {cfg.L} layers x {H} heads x d{d}, batch {B}, prompt {T} "
                               f"(positions {q_start}..{T - 1} after the membership decision), clusters/layer "
                               f"{sorted(set(ks_all))}, membership drawn ({cfg.membership if cfg.membership == 'skewed' else 'uniform'}), "
                               f"{n_res} layers resident and visited in turn",
                   "layers": cfg.L, "heads": H, "head_dim": d, "batch": B, "prompt": T},
        "roofline": roof,
        "useful_TFLOPs_whole_step": flops / (ms * 1e-3) / 1e12,
        "host_wall_ms_per_step": wall_ms,
    }
    if dense_ms is not None:
        result["dense_mha"] = {"ms_per_step": dense_ms, "TFLOPs": dense_flops / (dense_ms * 1e-3) / 1e12,
                               "speedup_clustered_over_dense": dense_ms / ms,
                               "ideal_speedup_by_flops": dense_flops / flops}
    if not args.no_cpu_baseline:
        from oracle import chai_oracle as O
        L = layers[-1]
        clustered_step()
        torch.cuda.synchronize()

        def run_oracle(nb, rows):
            qs = T - rows
            h2c, rep = L.h2c[:nb].cpu().numpy(), L.rep[:nb].cpu().numpy()
            qh = W.torch_to_host_bits(L.q[:nb, :, Tq - rows:])
            kh, vh = W.torch_to_host_bits(L.kfull[:nb]), W.torch_to_host_bits(L.v[:nb])
            t0 = time.perf_counter()
            ref = O.clustered_prefill(qh, kh, vh, h2c, rep, qs, cfg.scale)
            dt = time.perf_counter() - t0
            got = L.out[:nb, :, Tq - rows:].cpu().numpy().astype(np.float64)
            err = float((np.abs(got - ref).max(-1) / np.abs(ref).max(-1)).max())
            return dt, err, nb * sum(qs + i + 1 for i in range(rows)) * (L.k + H)

        # a short calibration run sizes the sample for about 12 s of oracle time: the last `rows` query rows
        # (the most expensive ones) of `nb` batch rows of one layer
        dt0, _, _ = run_oracle(1, min(48, Tq))
        per_row = max(dt0 / min(48, Tq), 1e-6)
        rows = max(min(Tq, int(12.0 / per_row)), 1)
        nb = min(B, max(int(12.0 / (per_row * Tq * 0.55)), 1)) if rows == Tq else 1
        dt, err, pairs_s = run_oracle(nb, rows)
        step_s = dt * sum(pairs * B * (k + H) for k in ks_all) / pairs_s
        result["cpu_baseline"] = {"value": B * Tq / step_s, "unit": "tokens/s", "cores": O.num_threads(),
                                  "kind": "oracle",
                                  "sample": f"last {rows} of {Tq} query rows of {nb} of {B} batch rows of one layer "
                                            f"({dt:.1f} s of oracle time), scaled by (query, key, head) count to "
                                            f"all rows, batch rows and layers",
                                  "parity_worst_normwise_err": err}
    print(json.dumps(result))


def shared_v_main(args, cfg, torch, C, W):
    """Decode step of the ablation that prunes values too (every head takes its representative's V): both caches
    compact, k streams each.  Priced against the HBM roofline like the headline path, and against the method
    proper (own V) on the same layers."""
    import numpy as np
    B, H, d, T, e = cfg.B, cfg.H, cfg.d, cfg.T, cfg.elem_bytes
    layers, _ = build_layers(cfg, W, C, torch, keep_full_k=False)
    vcs = []
    for L in layers:
        vc = torch.empty_like(L.kc)
        C.chai_compact_kcache(L.v, L.rep, vc, T)
        vcs.append(vc)
    ws = C.alloc_workspace(B, H, max(cfg.ks), T, d, cfg.dtype)

    def shared_step():
        for L, vc in zip(layers, vcs):
            C.chai_decode_attention_shared_v(L.q, L.kc, vc, L.h2c, L.rep, T, cfg.scale, L.out, ws)

    def own_v_step():
        for L in layers:
            C.chai_decode_attention(L.q, L.kc, L.v, L.h2c, L.rep, T, cfg.scale, L.out, ws)

    own_ms, _ = timed_steps(own_v_step, max(args.steps // 2, 3), args.warmup, torch)
    ms, wall_ms = timed_steps(shared_step, args.steps, args.warmup, torch)
    alg = sum(2 * B * L.k * T * d * e + B * L.k * d * e + 2 * B * H * 4 + B * H * d * 4 for L in layers)
    ach = alg / (ms * 1e-3) / 1e9
    result = {
        "metric": "decode-attn tokens/s of the ablation with shared values + achieved HBM GB/s vs peak",
        "value": B / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == W.BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}, values pruned as well: {cfg.L} layers x {H} heads x d{d}, batch {B}, "
                               f"context {T}, clusters/layer {sorted(set(cfg.ks))}, membership {cfg.membership}",
                   "layers": cfg.L, "heads": H, "head_dim": d, "batch": B, "context": T},
        "roofline": {"bound": "hbm", "kernel": "whole call (score, value and member-combine kernels)",
                     "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                     "traffic": None, "bytes_per_step": alg},
        "host_wall_ms_per_step": wall_ms,
        "own_values": {"ms_per_step": own_ms, "speedup_shared_over_own": own_ms / ms,
                       "ideal_speedup_by_bytes": cfg.clustered_bytes_per_step() / alg},
    }
    if not args.no_cpu_baseline:
        from oracle import chai_oracle as O
        shared_step()
        torch.cuda.synchronize()
        n_s = min(len(layers), 16)
        idx = sorted(set(int(round(i * (len(layers) - 1) / max(n_s - 1, 1))) for i in range(n_s)))
        dt, err = 0.0, 0.0
        for li in idx:
            L, vc = layers[li], vcs[li]
            rep, h2c = L.rep.cpu().numpy(), L.h2c.cpu().numpy()
            # full caches for the oracle: it reads only the representatives' rows (pinned), the rest stays zero
            kf = np.zeros((B, H, T, d), np.uint16 if cfg.dtype == W.BF16 else np.float32)
            vf = np.zeros_like(kf)
            kc_h, vc_h = W.torch_to_host_bits(L.kc[:, :, :T]), W.torch_to_host_bits(vc[:, :, :T])
            for b in range(B):
                for j in range(L.k):
                    if rep[b, j] >= 0:
                        kf[b, rep[b, j]], vf[b, rep[b, j]] = kc_h[b, j], vc_h[b, j]
            qh = W.torch_to_host_bits(L.q)
            t0 = time.perf_counter()
            ref = O.shared_v_decode(qh, kf, vf, h2c, rep, T, cfg.scale)
            dt += time.perf_counter() - t0
            got = L.out.cpu().numpy().astype(np.float64)
            err = max(err, float((np.abs(got - ref).max(-1) / np.abs(ref).max(-1)).max()))
        dt /= len(idx)
        result["cpu_baseline"] = {"value": B / (dt * cfg.L), "unit": "tokens/s", "cores": O.num_threads(),
                                  "kind": "oracle",
                                  "sample": f"every batch row of {len(idx)} of {cfg.L} layers ({dt * len(idx):.1f} s of "
                                            f"oracle time; it attends per head, so its cost does not depend on "
                                            f"the cluster count), scaled to all layers",
                                  "parity_worst_normwise_err": err}
    print(json.dumps(result))


def project_main(args, cfg, torch, C, W):
    """Query/key projections of the representatives for a block of prompt tokens (positions 5..T-1 of every batch
    row), all layers: the share of W_Q and W_K that clustered attention needs.  Dense baseline: the same kernel
    with every head its own representative (the full projections)."""
    import numpy as np
    B, H, d, T = cfg.B, cfg.H, cfg.d, cfg.T
    D = H * d
    pos0, Tn = W.N_TOK, T - W.N_TOK
    n_res = min(cfg.L, 4)
    layers = []
    for l in range(n_res):
        k = cfg.ks[(l * cfg.L) // n_res if cfg.L > n_res else l]
        seed = cfg.seed * 6007 + l
        L = Layer()
        L.k = k
        g = W.rng(cfg.seed, l, "member")
        _, rep = (W.sized_membership(g, B, H, cfg.sizes) if cfg.membership == "skewed"
                  else W.random_membership(g, B, H, k))
        L.rep = W.host_to_torch(rep)
        L.q = W.device_normal((B, Tn, D), cfg.dtype, seed + 1)                        # activations
        L.kfull = (W.device_normal((H * d, D), cfg.dtype, seed + 2) * 0.05).to(torch.bfloat16)     # w_q
        L.v = (W.device_normal((H * d, D), cfg.dtype, seed + 3) * 0.05).to(torch.bfloat16)         # w_k
        L.kc = torch.empty((B, k, T, d), dtype=torch.bfloat16, device="cuda")
        layers.append(L)
    q_out = torch.empty((B, H, Tn, d), dtype=torch.bfloat16, device="cuda")
    k_all = torch.empty((B, H, T, d), dtype=torch.bfloat16, device="cuda")
    ident = torch.arange(H, dtype=torch.int32, device="cuda").repeat(B, 1).contiguous()
    ks_all = [layers[(l * n_res) // cfg.L].k for l in range(cfg.L)]

    def clustered_step():
        for l in range(cfg.L):
            L = layers[(l * n_res) // cfg.L]
            C.chai_project_qk(L.q, L.kfull, L.v, L.rep, q_out, L.kc, pos0)

    def dense_step():
        for l in range(cfg.L):
            L = layers[(l * n_res) // cfg.L]
            C.chai_project_qk(L.q, L.kfull, L.v, ident, q_out, k_all, pos0)

    steps, warmup = max(args.steps // 4, 2), max(args.warmup // 2, 1)
    dense_ms = None
    if not args.no_dense:
        dense_ms, _ = timed_steps(dense_step, max(steps // 2, 1), warmup, torch)
    ms, wall_ms = timed_steps(clustered_step, steps, warmup, torch)
    layer_flops = {k: 2.0 * Tn * D * (2 * k * d) * B for k in set(ks_all)}
    flops = sum(layer_flops[k] for k in ks_all)
    dense_flops = 2.0 * Tn * D * (2 * H * d) * B * cfg.L
    hev = HipEvents()
    recs = {}
    for _ in range(max(steps // 2, 1)):
        for l in range(cfg.L):
            L = layers[(l * n_res) // cfg.L]
            e0, e1 = hev.create(), hev.create()
            C.chai_project_qk_timed(L.q, L.kfull, L.v, L.rep, q_out, L.kc, pos0, start_event=e0, stop_event=e1)
            recs.setdefault(L.k, []).append((e0, e1))
    torch.cuda.synchronize()
    kern = {k: sum(hev.elapsed_ms(a, b) for a, b in v) / len(v) for k, v in recs.items()}
    hev.close()
    k_dom = max(set(ks_all), key=ks_all.count)
    ach = layer_flops[k_dom] / (kern[k_dom] * 1e-3) / 1e12
    result = {
        "metric": "prompt tokens/s through the query/key projections of the representatives (all layers)",
        "value": B * Tn / (ms * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name} projection: {cfg.L} layers, model width {D} ({H} heads x d{d}), batch {B}, "
                               f"{Tn} prompt tokens per row (positions {pos0}..{T - 1}), clusters/layer "
                               f"{sorted(set(ks_all))}, {n_res} layers resident and visited in turn",
                   "layers": cfg.L, "heads": H, "head_dim": d, "batch": B, "prompt": T},
        "roofline": {"bound": "mfma", "kernel": f"project_kernel, layers with {k_dom} clusters", "achieved": ach,
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": ach / 2500.0,
                     "traffic": read_traffic(cfg.name, "project_kernel") if T == W.CONFIGS[cfg.name].T else None,
                     "avg_launch_ms": kern[k_dom], "flops_per_launch": layer_flops[k_dom],
                     "kernel_ms_by_clusters": {str(k): v for k, v in sorted(kern.items())}},
        "TFLOPs_whole_step": flops / (ms * 1e-3) / 1e12,
        "host_wall_ms_per_step": wall_ms,
    }
    ceil_tf = mfma_ceiling(layers[-1].kfull, C, torch)
    result["roofline"]["mfma_ceiling"] = {"TFLOPs": ceil_tf, "frac_of_peak": ceil_tf / 2500.0,
                                          "kernel_frac_of_ceiling": ach / ceil_tf,
                                          "how": "matrix pipe alone on the workload's weight data (chai_mfma_rate_probe)"}
    if dense_ms is not None:
        result["dense_projection"] = {"ms_per_step": dense_ms, "TFLOPs": dense_flops / (dense_ms * 1e-3) / 1e12,
                                      "speedup_pruned_over_dense": dense_ms / ms,
                                      "ideal_speedup_by_flops": dense_flops / flops}
    if not args.no_cpu_baseline:
        from oracle import chai_oracle as O
        L = layers[-1]
        C.chai_project_qk(L.q, L.kfull, L.v, L.rep, q_out, L.kc, pos0)
        torch.cuda.synchronize()
        wq, wk = W.torch_to_host_bits(L.kfull), W.torch_to_host_bits(L.v)
        rep = L.rep.cpu().numpy()

        def run_oracle(rows):
            xh = W.torch_to_host_bits(L.q[:, Tn - rows:])
            t0 = time.perf_counter()
            q_ref, k_ref = O.project_qk(xh, wq, wk, rep, d)
            dt = time.perf_counter() - t0
            got_k = W.bf16_bits_to_f32(W.torch_to_host_bits(L.kc[:, :, T - rows:T])).astype(np.float64)
            used = rep >= 0
            err = float(np.max(np.abs(got_k[used] - k_ref[used]) /
                               np.maximum(np.abs(k_ref[used]).max(-1, keepdims=True), 1e-30)))
            return dt, err

        dt0, _ = run_oracle(min(8, Tn))                      # calibration, then about 10 s of oracle time
        rows = max(min(Tn, int(10.0 / max(dt0 / min(8, Tn), 1e-6))), 1)
        dt, err = run_oracle(rows)
        step_s = dt * (Tn / rows) * sum(ks_all) / L.k
        result["cpu_baseline"] = {"value": B * Tn / step_s, "unit": "tokens/s", "cores": O.num_threads(), "kind": "oracle",
                                  "sample": f"last {rows} of {Tn} tokens of every batch row of one layer ({dt:.1f} s of "
                                            f"oracle time), scaled by token and cluster count to all layers",
                                  "parity_worst_normwise_err": err,
                                  "parity_note": "outputs are bf16: one rounding, up to 2^-8 of an element"}
    print(json.dumps(result))


def decode_bench(cfg, args, torch, C, W, steps, warmup, want_cpu, want_dense=True, want_phase=True, want_ceiling=True,
                 want_sampled_parity=False):
    """Time one configuration's decode step (the attention of all layers for one token of every batch row) and
    return the result record."""
    B, H, d, T = cfg.B, cfg.H, cfg.d, cfg.T
    layers, t_member = build_layers(cfg, W, C, torch, keep_full_k=want_dense or want_cpu or want_sampled_parity)
    ws = C.alloc_workspace(B, H, H, T, d, cfg.dtype)       # sized for the dense call; serves every layer

    def clustered_step():
        for L in layers:
            C.chai_decode_attention(L.q, L.kc, L.v, L.h2c, L.rep, T, cfg.scale, L.out, ws)

    def dense_step():
        for L in layers:
            C.chai_dense_decode_attention(L.q, L.kfull, L.v, T, cfg.scale, L.out, ws)

    dense_ms = None
    if want_dense:
        dense_ms, _ = timed_steps(dense_step, max(steps // 2, 3), warmup, torch)
    ms, wall_ms = timed_steps(clustered_step, steps, warmup, torch)

    alg_bytes = cfg.clustered_bytes_per_step()
    result = {
        "metric": "clustered decode-attn tokens/s + achieved HBM GB/s vs peak, vs dense MHA",
        "value": B / (ms * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == W.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.L} layers x {H} heads x d{d}, batch {B}, context {T}, "
                               f"clusters/layer {sorted(set(cfg.ks))}, membership {cfg.membership}",
                   "layers": cfg.L, "heads": H, "head_dim": d, "batch": B, "context": T},
        "algorithmic_GBps": alg_bytes / (ms * 1e-3) / 1e9,
        "frac_of_hbm_peak": alg_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "algorithmic_bytes_per_step": alg_bytes,
        "host_wall_ms_per_step": wall_ms,
        "membership_and_compaction_s": t_member,
        "k_cache_bytes_saved": cfg.k_bytes_saved(),
        "k_cache_fraction_saved": cfg.k_bytes_saved() / (cfg.L * B * H * T * d * cfg.elem_bytes),
    }
    if dense_ms is not None:
        result["dense_mha"] = {"ms_per_step": dense_ms, "tokens_per_s": B / (dense_ms * 1e-3),
                               "GBps": cfg.dense_bytes_per_step() / (dense_ms * 1e-3) / 1e9,
                               "speedup_clustered_over_dense": dense_ms / ms,
                               "ideal_speedup_by_bytes": cfg.dense_bytes_per_step() / alg_bytes}

    if want_phase:
        ph = phase_timing(layers, cfg, ws, C, torch, max(min(steps, 10), 2))
        e = cfg.elem_bytes
        # dominant kernel: the value kernel (streams B*H*T*d elements of V per launch, the same for every layer)
        v_ms = sum(v for _, v in ph.values()) / len(ph)
        v_bytes = B * H * T * d * e + B * H * d * 4
        s_bytes = sum(B * L.k * T * d * e for L in layers) / len(layers)
        s_ms = sum(sv for sv, _ in ph.values()) / len(ph)
        ach = v_bytes / (v_ms * 1e-3) / 1e9
        result["roofline"] = {"bound": "hbm", "kernel": "value_kernel", "achieved": ach, "peak": HBM_PEAK_GBS,
                              "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                              "traffic": read_traffic(cfg.name) if T == W.CONFIGS[cfg.name].T else None,
                              "bytes_per_launch": v_bytes, "avg_launch_ms": v_ms}
        result["score_kernel"] = {"avg_launch_ms": s_ms, "avg_bytes_per_launch": s_bytes,
                                  "achieved_GBps": s_bytes / (s_ms * 1e-3) / 1e9,
                                  "frac": s_bytes / (s_ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        if want_ceiling:
            ceiling = read_ceiling(layers, C, torch)
            result["read_ceiling"] = {"GBps": ceiling, "frac_of_peak": ceiling / HBM_PEAK_GBS,
                                      "value_kernel_frac_of_ceiling": ach / ceiling,
                                      "step_frac_of_ceiling": result["algorithmic_GBps"] / ceiling,
                                      "how": "bare streaming read of the value caches (chai_stream_read_probe), median launch"}

    if want_cpu or want_sampled_parity:
        clustered_step()
        torch.cuda.synchronize()
    if want_cpu:
        result["cpu_baseline"] = cpu_baseline(cfg, layers, W, torch)
    if want_sampled_parity:
        result["parity_sampled"] = sampled_parity(cfg, layers, W, torch)
    del layers, ws
    torch.cuda.empty_cache()
    return result


def q8_bench(cfg, args, torch, C, W, steps, warmup, want_parity=True):
    """Decode step over QUANTISED caches (8-bit floating point codes, one fp32 scale per cached row) of the same
    configuration: the caches are built as for the bf16 path, quantised by the library, and attended to through
    chai_decode_attention_q8.  Algorithmic bytes are the method's own for this storage: 132 bytes per cached row."""
    import numpy as np
    B, H, d, T = cfg.B, cfg.H, cfg.d, cfg.T
    layers, _ = build_layers(cfg, W, C, torch, keep_full_k=want_parity)
    q8 = []
    for L in layers:
        k8, ks = C.chai_quantize_rows(L.kc)
        v8, vs = C.chai_quantize_rows(L.v)
        q8.append((k8, ks, v8, vs))
        L.kc = None
        if not want_parity:
            L.v = None
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    ws = torch.empty((C.chai_decode_q8_workspace_bytes(B, H, max(cfg.ks), T),), dtype=torch.uint8, device="cuda")

    def step():
        for L, (k8, ks, v8, vs) in zip(layers, q8):
            C.chai_decode_attention_q8(L.q, k8, ks, v8, vs, L.h2c, L.rep, T, cfg.scale, L.out, ws)

    ms, wall_ms = timed_steps(step, steps, warmup, torch)
    row_bytes = d + 4
    alg = sum(B * (L.k + H) * T * row_bytes + B * L.k * d * cfg.elem_bytes + 2 * B * H * 4 + B * H * d * 4 for L in layers)
    hev = HipEvents()
    recs = []
    for _ in range(max(min(steps, 10), 2)):
        for L, (k8, ks, v8, vs) in zip(layers, q8):
            e = [hev.create() for _ in range(4)]
            C.chai_decode_attention_q8_timed(L.q, k8, ks, v8, vs, L.h2c, L.rep, T, cfg.scale, L.out, ws,
                                             score_events=(e[0], e[1]), value_events=(e[2], e[3]))
            recs.append(e)
    torch.cuda.synchronize()
    s_ms = sum(hev.elapsed_ms(e[0], e[1]) for e in recs) / len(recs)
    v_ms = sum(hev.elapsed_ms(e[2], e[3]) for e in recs) / len(recs)
    hev.close()
    v_bytes = B * H * T * row_bytes + B * H * d * 4
    ach = v_bytes / (v_ms * 1e-3) / 1e9
    rec = {"storage": "E4M3 codes + one fp32 scale per cached row (132 bytes per row instead of 256)",
           "workload": f"{cfg.name}: {cfg.L} layers x {H} heads x d{d}, batch {B}, context {T}",
           "tokens_per_s": B / (ms * 1e-3), "ms_per_step": ms, "algorithmic_bytes_per_step": alg,
           "algorithmic_GBps": alg / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "roofline": {"bound": "hbm", "kernel": "value_kernel (8-bit rows)", "achieved": ach, "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": read_traffic(cfg.name, "value_kernel_q8") if T == W.CONFIGS[cfg.name].T else None, "bytes_per_launch": v_bytes,
                        "avg_launch_ms": v_ms},
           "score_kernel_ms": s_ms, "host_wall_ms_per_step": wall_ms}
    if want_parity:
        # dense multi-head attention over quantised caches: the same kernels with every head its own cluster
        # (identity maps) over the quantised FULL key cache
        ident_h2c = torch.arange(H, dtype=torch.int32, device="cuda").repeat(B, 1).contiguous()
        ws_d = torch.empty((C.chai_decode_q8_workspace_bytes(B, H, H, T),), dtype=torch.uint8, device="cuda")
        n_dense = len(layers)
        kq_full = [C.chai_quantize_rows(layers[i].kfull) for i in range(n_dense)]

        def dense_step():
            for i in range(n_dense):
                L, (k8, ks, v8, vs) = layers[i], q8[i]
                C.chai_decode_attention_q8(L.q, kq_full[i][0], kq_full[i][1], v8, vs, ident_h2c, ident_h2c, T, cfg.scale,
                                           L.out, ws_d)

        d_ms, _ = timed_steps(dense_step, max(steps // 2, 3), warmup, torch)
        d_ms *= len(layers) / n_dense
        dense_bytes = len(layers) * (2 * B * H * T * row_bytes)
        rec["dense_mha_q8"] = {"ms_per_step": d_ms, "tokens_per_s": B / (d_ms * 1e-3),
                               "GBps": dense_bytes / (d_ms * 1e-3) / 1e9, "speedup_clustered_over_dense": d_ms / ms,
                               "ideal_speedup_by_bytes": dense_bytes / alg,
                               "how": "same kernels, identity maps, quantised full key cache, every layer"}
        del kq_full, ws_d
        from oracle import chai_oracle as O
        step()
        torch.cuda.synchronize()
        g = np.random.default_rng(cfg.seed + 8)
        worst, codes_equal = 0.0, True
        for li in sorted(set([0, len(layers) - 1])):
            L, (k8, ks, v8, vs) = layers[li], q8[li]
            h2c, rep = L.h2c.cpu().numpy(), L.rep.cpu().numpy()
            for _ in range(4):
                b, h = int(g.integers(B)), int(g.integers(H))
                c = int(h2c[b, h])
                r = int(rep[b, c])
                # the oracle quantises the representative's FULL-cache key stream and this head's value stream itself
                kq, ksq = O.quantize_rows(W.torch_to_host_bits(L.kfull[b, r, :T]))
                vq, vsq = O.quantize_rows(W.torch_to_host_bits(L.v[b, h, :T]))
                codes_equal = (codes_equal and np.array_equal(kq, k8[b, c, :T].cpu().numpy())
                               and np.array_equal(ksq, ks[b, c, :T].cpu().numpy())
                               and np.array_equal(vq, v8[b, h, :T].cpu().numpy())
                               and np.array_equal(vsq, vs[b, h, :T].cpu().numpy()))
                qr = W.torch_to_host_bits(L.q[b, r])
                ref = O.clustered_decode_q8(np.stack([qr, qr * 0])[None], np.stack([kq, kq * 0])[None],
                                            np.stack([ksq, ksq * 0])[None], np.stack([vq * 0, vq])[None],
                                            np.stack([vsq * 0, vsq])[None], np.zeros((1, 2), np.int32),
                                            np.zeros((1, 1), np.int32), T, cfg.scale)[0, 1]
                got = L.out[b, h].cpu().numpy().astype(np.float64)
                worst = max(worst, float(np.abs(got - ref).max() / np.abs(ref).max()))
        rec["parity"] = {"worst_normwise_err_vs_oracle_on_same_codes": worst, "codes_and_scales_equal_oracle": codes_equal,
                         "sampled_heads": 8}
        if worst > 2e-5 or not codes_equal:
            raise RuntimeError(f"quantised decode parity failed: {rec['parity']}")
    del layers, q8, ws
    torch.cuda.empty_cache()
    return rec


def e2e_bench(cfg, args, torch, C, W, steps_timed=2):
    """The end-to-end flow of the OPT-66B-shaped configuration, all layers at full size: caches hold a prompt of
    cfg.prompt tokens -> score features of the first five positions -> k-means -> K-cache compaction (timed: the
    clustering overhead the paper counts into the time to first token) -> cfg.decode_steps decode steps with
    cache growth through chai_decode_step (append folded into the attention kernels), once from the end of the
    prompt (contexts prompt+1 ...) and once ending at the cache capacity (the 2048-token point).  Parity inside the
    run: the oracle on sampled (batch row, head) pairs at the first, the middle and the last step, fed the FULL
    key cache of the prompt plus the appended rows, and byte equality of the grown caches with chai_append_kv."""
    import numpy as np
    from oracle import chai_oracle as O
    B, H, d, L, P, S, T_cap = cfg.B, cfg.H, cfg.d, cfg.L, cfg.prompt, cfg.decode_steps, cfg.T_cap
    k = cfg.ks[0]
    dev = "cuda"
    bf = torch.bfloat16
    kfull, v, kc, q5, init, qs, kn, vn, h2c, rep, ncl, its, feat, out = ([] for _ in range(14))
    for l in range(L):
        seed = cfg.seed * 200003 + l * 31
        kfull.append(W.device_normal((B, H, P, d), cfg.dtype, seed + 1, dev))          # the prompt's keys, every head
        v.append(W.device_normal((B, H, T_cap, d), cfg.dtype, seed + 2, dev))
        kc.append(W.device_normal((B, k, T_cap, d), cfg.dtype, seed + 3, dev))         # rows >= P: "decoded earlier"
        q5.append(W.device_normal((B, H, W.N_TOK, d), cfg.dtype, seed + 4, dev))
        qs.append(W.device_normal((S, B, H, d), cfg.dtype, seed + 5, dev))
        kn.append(W.device_normal((S, B, H, d), cfg.dtype, seed + 6, dev))
        vn.append(W.device_normal((S, B, H, d), cfg.dtype, seed + 7, dev))
        init.append(W.host_to_torch(W.distinct_heads(W.rng(cfg.seed, l, "init"), B, H, k), dev))
        h2c.append(torch.empty((B, H), dtype=torch.int32, device=dev))
        rep.append(torch.empty((B, k), dtype=torch.int32, device=dev))
        ncl.append(torch.empty((B,), dtype=torch.int32, device=dev))
        its.append(torch.empty((B,), dtype=torch.int32, device=dev))
        feat.append(torch.empty((B, H, W.N_TOK * W.N_TOK), dtype=torch.float32, device=dev))
        out.append(torch.empty((B, H, d), dtype=torch.float32, device=dev))
    ws = C.alloc_workspace(B, H, k, T_cap, d, cfg.dtype)

    # ---- phase 1: membership and compaction of every layer (nothing allocated inside the timed region)
    def membership():
        for l in range(L):
            C.chai_score_features(q5[l], kfull[l], W.N_TOK, cfg.scale, feat=feat[l])
            C.chai_assign_clusters(feat[l], init[l], head_to_cluster=h2c[l], rep_heads=rep[l], n_clusters=ncl[l],
                                   iters=its[l])
            C.chai_compact_kcache(kfull[l], rep[l], kc[l], P)
    member_ms, _ = timed_steps(membership, 3, 1, torch)

    # ---- phase 2: decode with cache growth
    def run_pass(start, step_list=None):
        for st in (range(S) if step_list is None else step_list):
            T = start + st + 1
            for l in range(L):
                C.chai_decode_step(qs[l][st], kn[l][st], vn[l][st], kc[l], v[l], h2c[l], rep[l], T, cfg.scale, out[l], ws)

    record = {"flow": f"{L} layers x {H} heads, batch {B}: prompt {P} -> features of {W.N_TOK} positions -> k-means "
                      f"k={k} -> compaction -> {S} x chai_decode_step with cache growth",
              "membership_and_compaction_ms": member_ms,
              "membership_and_compaction_ms_per_layer": member_ms / L,
              "kmeans_passes_max": int(max(int(t.max()) for t in its)),
              "k_cache_fraction_saved": (H - k) / H}

    # parity pass (eager, untimed): sampled layers keep reference caches grown with chai_append_kv
    sample_layers = sorted(set(int(round(i * (L - 1) / 3)) for i in range(4)))
    g = np.random.default_rng(cfg.seed + 7)
    for name, start in (("from_prompt", P), ("to_capacity", T_cap - S)):
        kc_ref = {l: kc[l].clone() for l in sample_layers}
        v_ref = {l: v[l].clone() for l in sample_layers}
        worst, checked = 0.0, 0
        marks = sorted(set([0, S // 2 - 1, S - 1]))
        prev = 0
        for mark in marks:
            run_pass(start, range(prev, mark + 1))
            torch.cuda.synchronize()
            prev = mark + 1
            T = start + mark + 1
            for l in sample_layers:
                h2c_h, rep_h = h2c[l].cpu().numpy(), rep[l].cpu().numpy()
                for _ in range(3):
                    b, h = int(g.integers(B)), int(g.integers(H))
                    c = int(h2c_h[b, h])
                    r = int(rep_h[b, c])
                    # the representative's FULL key stream: prompt rows of the uncompacted cache, rows the cache
                    # held before this pass, then the rows appended so far
                    k_rows = np.concatenate([W.torch_to_host_bits(kfull[l][b, r]),
                                             W.torch_to_host_bits(kc_ref[l][b, c, P:start]),
                                             W.torch_to_host_bits(kn[l][:mark + 1, b, r])])
                    v_rows = np.concatenate([W.torch_to_host_bits(v_ref[l][b, h, :start]),
                                             W.torch_to_host_bits(vn[l][:mark + 1, b, h])])
                    qr = W.torch_to_host_bits(qs[l][mark, b, r])
                    ref = O.clustered_decode(np.stack([qr, qr * 0])[None], np.stack([k_rows, k_rows * 0])[None],
                                             np.stack([v_rows * 0, v_rows])[None], np.zeros((1, 2), np.int32),
                                             np.zeros((1, 1), np.int32), T, cfg.scale)[0, 1]
                    got = out[l][b, h].cpu().numpy().astype(np.float64)
                    worst = max(worst, float(np.abs(got - ref).max() / np.abs(ref).max()))
                    checked += 1
        # grown caches against the stand-alone append, byte for byte
        caches_equal = True
        for l in sample_layers:
            for st in range(S):
                C.chai_append_kv(kn[l][st], vn[l][st], rep[l], kc_ref[l], v_ref[l], start + st)
            torch.cuda.synchronize()
            caches_equal = caches_equal and torch.equal(kc_ref[l], kc[l]) and torch.equal(v_ref[l], v[l])
        del kc_ref, v_ref
        if worst > 2e-5 or not caches_equal:
            raise RuntimeError(f"end-to-end parity failed ({name}): worst {worst:.3g}, caches equal {caches_equal}")

        # timed passes: eager, then one HIP graph of the whole pass (host launch cost out of the way)
        ev_ms, wall = timed_steps(lambda: run_pass(start), steps_timed, 1, torch)
        graph_ms = None
        try:
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(graph, stream=side):
                    run_pass(start)
            torch.cuda.current_stream().wait_stream(side)
            graph_ms, _ = timed_steps(graph.replay, steps_timed, 1, torch)
            del graph
        except Exception as exc:      # capture not supported for these launches: the eager figure stands
            record.setdefault("graph_note", f"graph capture failed: {type(exc).__name__}: {exc}"[:200])
        best = min(ev_ms, graph_ms) if graph_ms is not None else ev_ms
        alg = sum(cfg.clustered_bytes_per_step(start + st + 1) + B * (k + H) * d * cfg.elem_bytes * 2 * L
                  for st in range(S))
        record[name] = {"contexts": [start + 1, start + S], "decode_steps": S,
                        "ms_total_eager": ev_ms, "ms_total_graph": graph_ms,
                        "ms_per_step": best / S, "tokens_per_s": B * S / (best * 1e-3),
                        "algorithmic_GBps": alg / (best * 1e-3) / 1e9,
                        "frac_of_hbm_peak": alg / (best * 1e-3) / 1e9 / HBM_PEAK_GBS,
                        "parity": {"worst_normwise_err": worst, "sampled_heads": checked,
                                   "at_steps": [m + 1 for m in marks], "layers": sample_layers,
                                   "grown_caches_equal_chai_append_kv": caches_equal,
                                   "key_source": "full prompt key cache + appended rows"}}
    p, c = record["from_prompt"], record["to_capacity"]
    record["time_to_first_token_overhead_vs_decode_step"] = member_ms / p["ms_per_step"]
    del kfull, v, kc, qs, kn, vn
    torch.cuda.empty_cache()
    return record


def brief(r):
    """The per-configuration figures that go next to the headline record."""
    out = {"workload": r["config"]["workload"], "tokens_per_s": r["value"], "ms_per_step": r["ms_per_step"],
           "algorithmic_GBps": r["algorithmic_GBps"], "frac_of_hbm_peak": r["frac_of_hbm_peak"], "dtype": r["dtype"]}
    if "roofline" in r:
        out["value_kernel_frac"] = r["roofline"]["frac"]
        out["value_kernel_ms"] = r["roofline"]["avg_launch_ms"]
        out["value_kernel_traffic"] = r["roofline"]["traffic"]
        out["score_kernel_frac"] = r["score_kernel"]["frac"]
        out["score_kernel_ms"] = r["score_kernel"]["avg_launch_ms"]
    if "dense_mha" in r:
        out["dense_ms_per_step"] = r["dense_mha"]["ms_per_step"]
        out["speedup_over_dense"] = r["dense_mha"]["speedup_clustered_over_dense"]
        out["ideal_speedup_by_bytes"] = r["dense_mha"]["ideal_speedup_by_bytes"]
    out["k_cache_fraction_saved"] = r["k_cache_fraction_saved"]
    if "parity_sampled" in r:
        out["parity_sampled"] = r["parity_sampled"]
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import dataclasses

    import torch

    import paper_2403_08058_amd as C
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)

    cfg = W.CONFIGS[args.config]
    if args.context:
        cfg = dataclasses.replace(cfg, T=args.context, T_cap=max(cfg.T_cap, args.context))
    if args.mode == "prefill":
        prefill_main(args, cfg, torch, C, W)
        return
    if args.mode == "shared-v":
        shared_v_main(args, cfg, torch, C, W)
        return
    if args.mode == "project":
        project_main(args, cfg, torch, C, W)
        return
    if args.mode == "q8":
        r = q8_bench(cfg, args, torch, C, W, args.steps, args.warmup, want_parity=not args.no_cpu_baseline)
        r.update({"metric": "clustered decode-attn tokens/s over 8-bit quantised K,V caches", "value": r["tokens_per_s"],
                  "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True,
                  "scaling": "weak", "vs_baseline": None, "dtype": "e4m3 codes, f32 accumulate", "data": "synthetic",
                  "config": {"workload": r["workload"]}})
        print(json.dumps(r))
        return
    if args.mode == "e2e":
        print(json.dumps({"metric": "end-to-end clustered decode with cache growth", "config": {"workload": cfg.name},
                          "e2e": e2e_bench(W.CONFIGS["cfg4"], args, torch, C, W)}))
        return

    result = decode_bench(cfg, args, torch, C, W, args.steps, args.warmup, want_cpu=not args.no_cpu_baseline,
                          want_dense=not args.no_dense, want_phase=not args.no_phase_timing)
    if args.config == "cfg4" and not args.context and not args.no_configs:
        result["e2e"] = e2e_bench(cfg, args, torch, C, W)

    # the other configurations next to the headline one (default run only): same code path, same step counts
    if args.config == "cfg2" and not args.context and not args.no_configs:
        others = {}
        for name in ("cfg1", "cfg3", "cfg4", "cfg5"):
            c = W.CONFIGS[name]
            time.sleep(args.settle)        # each configuration starts from an idle card, as a run of its own would
            r = decode_bench(c, args, torch, C, W, args.steps, args.warmup, want_cpu=False, want_dense=True,
                             want_phase=True, want_ceiling=False, want_sampled_parity=True)
            others[name] = brief(r)
        c4 = W.CONFIGS["cfg4"]
        time.sleep(args.settle)
        r640 = decode_bench(dataclasses.replace(c4, T=c4.prompt + c4.decode_steps), args, torch, C, W, args.steps,
                            args.warmup, want_cpu=False, want_dense=True, want_phase=True, want_ceiling=False)
        others["cfg4"]["fixed_context_640"] = brief(r640)
        others["cfg4"]["e2e"] = e2e_bench(c4, args, torch, C, W)
        result["configs"] = others
        result["configs_settle_s"] = args.settle
        time.sleep(args.settle)
        result["quantised_kv"] = q8_bench(cfg, args, torch, C, W, max(min(args.steps, 10), 2), 2)

    print(json.dumps(result))


if __name__ == "__main__":
    main()
