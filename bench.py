#!/usr/bin/env python3
"""Throughput of the Encode stage (ViT forward, V_m = E(I_m); paper section 3.1, Eq. 1) on one
MI355X: visual tokens per second, synthetic seeded inputs.

The headline workload is the largest single-GPU benchmark configuration, C5: the 45-layer
video encoder (hidden 3200, 25 heads x 128, MLP 12800, patch 14 x temporal 2, 3-D rotary) on
four clips of 16 frames at 448 x 448 -- 32 768 packed patch tokens -> 8192 visual tokens.  One
"step" is one epd_encode call: plan, patch embedding, all transformer blocks, final norm, 2x2
merge and projection, with the packed patches and weights already resident in HBM.  The other
bf16 configurations (C2, C3, C4) and the batch of the paper's Table 4_2 resolutions (T42) are
timed in the same run, briefly, and reported in the "others" block of the line.

Prints ONE JSON line on stdout; progress and the per-step tables go to stderr.
"""

from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
ROOT = os.path.dirname(os.path.abspath(__file__))


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class PowerSampler:
    """Board power while a region runs: a thread reads the GPU's hwmon power sensor (microwatts,
    /sys/class/drm/card*/device/hwmon/hwmon*/power1_input) every 20 ms.  Read-only; where the
    sensor is not readable the summary is None.  `cap_w` is the board's power limit from the
    same directory."""

    def __init__(self, period_s=0.02):
        import glob
        import threading
        self.path = next((f for f in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input")) if os.access(f, os.R_OK)), None)
        self.period, self.samples, self._stop = period_s, [], threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True) if self.path else None

    def _read(self, path):
        try:
            with open(path) as f:
                return int(f.read().strip()) / 1e6
        except (OSError, ValueError):
            return None

    def _run(self):
        while not self._stop.is_set():
            w = self._read(self.path)
            if w is not None:
                self.samples.append(w)
            self._stop.wait(self.period)

    def __enter__(self):
        if self._thread:
            self._thread.start()
        return self

    def __exit__(self, *exc):
        if self._thread:
            self._stop.set()
            self._thread.join()

    def summary(self, tail=0.75):
        if not self.samples:
            return None
        # the sensor is a moving average over a second or more: the first samples of a region still
        # hold what ran before it, so the mean is taken over the last `tail` of the samples
        body = self.samples[int(len(self.samples) * (1.0 - tail)):] or self.samples
        cap = self._read(os.path.join(os.path.dirname(self.path), "power1_cap"))
        return {"mean_w": sum(body) / len(body), "max_w": max(self.samples), "samples": len(self.samples), "cap_w": cap,
                "sensor": "hwmon power1_input, 20 ms period, mean over the last %.0f %% of the region" % (100 * tail)}


def host_cores():
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env))
    return cores


def parity_numbers(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    cos = (got * ref).sum(-1) / (np.linalg.norm(got, axis=-1) * np.linalg.norm(ref, axis=-1))
    rel = np.abs(got - ref).max(-1) / np.abs(ref).max(-1)
    return float(cos.min()), float(rel.max())


def cpu_baseline_full(cfg, gw, layers, patches, grid, gpu_out, n_items):
    """The CPU oracle, as it stands, on the first n_items items of the batch at full depth
    (configurations the oracle finishes in seconds)."""
    from oracle import vit_encode as O
    from paper_2601_11590_amd import workloads as W
    grids = [tuple(int(v) for v in g) for g in grid[:n_items]]
    T, Tm = W.num_tokens(grids), W.num_merged_tokens(grids, cfg.merge)
    cu1, g1 = W.metadata(grids)
    t0 = time.perf_counter()
    ref = O.encode(cfg, gw, layers, patches[:T], cu1, g1)
    dt = time.perf_counter() - t0
    cos, rel = parity_numbers(gpu_out[:Tm], ref)
    log("[bench] oracle on %d item(s), %d layers: %.2f s; GPU rows vs oracle: min cos %.6f, max rel %.3e" % (n_items, cfg.num_layers, dt, cos, rel))
    return {"value": Tm / dt, "unit": "visual tokens/s", "cores": host_cores(), "kind": "oracle",
            "sample": "first %d of the %d items (%d patch tokens -> %d visual tokens), all %d layers, fp64 NumPy, one run"
                      % (n_items, len(grid), T, Tm, cfg.num_layers),
            "seconds": dt, "parity_min_cos": cos, "parity_max_rel": rel}


def cpu_baseline_depth_sample(cfg, gw, layer0, patches, grid):
    """The CPU oracle, as it stands, on one item of the batch (the largest of at most 12 288
    tokens, else the smallest) with 0 and with 1 of the configuration's layers (a full-depth run
    takes the oracle tens of minutes); the rate at full depth is the linear extrapolation in
    depth, every layer having the same shape."""
    from oracle import vit_encode as O
    from paper_2601_11590_amd import workloads as W
    toks = [int(t) * int(h) * int(w) for t, h, w in grid]
    fits = [i for i, n in enumerate(toks) if n <= 12288]
    item = max(fits, key=lambda i: toks[i]) if fits else int(np.argmin(toks))
    g0 = [tuple(int(v) for v in grid[item])]
    T, Tm = W.num_tokens(g0), W.num_merged_tokens(g0, cfg.merge)
    first = sum(toks[:item])
    rows = patches[first:first + T]
    cu1, g1 = W.metadata(g0)
    t = time.perf_counter()
    O.encode(cfg.replace(num_layers=0), gw, [], rows, cu1, g1)
    t_l0 = time.perf_counter() - t
    t = time.perf_counter()
    O.encode(cfg.replace(num_layers=1), gw, [layer0], rows, cu1, g1)
    t_l1 = time.perf_counter() - t
    per_layer = max(t_l1 - t_l0, 1e-9)
    full = t_l0 + cfg.num_layers * per_layer
    log("[bench] oracle on item %d (%d tokens): %.2f s with 0 layers, %.2f s with 1 layer -> %.0f s extrapolated to %d layers"
        % (item, T, t_l0, t_l1, full, cfg.num_layers))
    return {"value": Tm / full, "unit": "visual tokens/s", "cores": host_cores(), "kind": "oracle",
            "sample": "item %d of %d (%d patch tokens -> %d visual tokens): the oracle timed once with 0 layers (%.2f s) and once "
                      "with 1 layer (%.2f s) of the %d; value = %d / (t0 + %d (t1 - t0)), a linear extrapolation in depth "
                      "(all layers have one shape), fp64 NumPy" % (item, len(grid), T, Tm, t_l0, t_l1, cfg.num_layers, Tm, cfg.num_layers),
            "seconds": t_l0 + t_l1, "extrapolated_full_depth_seconds": full}


def stored_rows_parity(name, gpu_out):
    """Full-depth parity against the oracle rows stored under tests/golden/ (C4, C5)."""
    path = os.path.join(ROOT, "tests", "golden", "%s_full_depth_rows.npz" % name.lower())
    if not os.path.exists(path):
        return None
    z = np.load(path, allow_pickle=False)
    rows, first = z["rows"], int(z["first_row_in_batch"])
    cos, rel = parity_numbers(gpu_out[first + rows], z["values"])
    log("[bench] %s full depth vs %d stored oracle rows: min cos %.6f, max rel %.3e" % (name, len(rows), cos, rel))
    return {"rows": int(len(rows)), "min_cos": cos, "max_rel": rel, "source": "tests/golden/%s" % os.path.basename(path)}


def flops_per_call(cfg, T, Tm, cu):
    D, F, L = cfg.hidden, cfg.mlp_dim, cfg.num_layers
    attn = L * sum(4.0 * float(cu[i + 1] - cu[i]) ** 2 * D for i in range(len(cu) - 1))
    return (2.0 * T * cfg.patch_dim * D + L * (8.0 * T * D * D + 4.0 * T * D * F) + attn
            + 2.0 * Tm * (cfg.merge ** 2 * D) * cfg.out_dim), attn


def stored_traffic(name, step):
    """HBM-side bytes per launch of `step` from the rocprofv3 --pmc summary under profiles/ (they
    cannot be collected in-process).  The summary carries the hash of the kernel sources it was
    measured on; a summary of other sources is not used."""
    from paper_2601_11590_amd import build as bld
    path = os.path.join(ROOT, "profiles", "%s_bench_hbm_traffic.txt" % name.lower())
    if not os.path.exists(path):
        return None, "no counter summary for %s under profiles/" % name
    val, stamp = None, None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == "SOURCE_HASH":
            stamp = parts[1]
        if len(parts) >= 3 and parts[0] == "TRAFFIC_BYTES_PER_LAUNCH" and parts[1] == step:
            val = float(parts[2])
    if stamp != bld.source_hash():
        return None, "profiles/%s was measured on other kernel sources (hash differs): dropped" % os.path.basename(path)
    return val, "profiles/%s" % os.path.basename(path)


def measure(name, steps, warmup, in_flight=1, layers_override=None, segments="item", keep_inputs=False, zero_data=False,
            gemm_tile=-1, attn_rows=0):
    """Times `steps` epd_encode calls of configuration `name`.  Returns a dict of results.
    zero_data: every weight and every input element is zero -- the same kernels and launches on
    operands that toggle no wires, which shows how much of the time on real data is the chip's
    power limit rather than the kernels' own pipelines (never the headline)."""
    import torch
    from paper_2601_11590_amd import binding as B, workloads as W
    cfg = W.CONFIGS[name]
    grids = W.grids_for(cfg)
    if layers_override is not None:
        cfg = cfg.replace(num_layers=layers_override)
    T, Tm = W.num_tokens(grids), W.num_merged_tokens(grids, cfg.merge)
    cu, grid = W.metadata(grids, segments)
    log("[bench] %s: %d items, %d segments, T=%d patch tokens -> %d visual tokens, L=%d" % (cfg.name, len(grids), len(cu) - 1, T, Tm, cfg.num_layers))
    t0 = time.perf_counter()
    gw = W.global_weights(cfg)
    patches = W.packed_patches(cfg, grids)
    layer0 = W.layer_weights(cfg, 0) if cfg.num_layers > 0 else None
    kept_layers = []
    if zero_data:
        gw = {k: np.zeros_like(v) for k, v in gw.items()}
        patches = np.zeros_like(patches)
        layer0 = {k: np.zeros_like(v) for k, v in layer0.items()} if layer0 else None

    def layer_stream():     # one layer at a time: 45 layers of C5 would be 22 GB of float32 on the host
        for l in range(cfg.num_layers):
            lw = layer0 if (l == 0 or zero_data) else W.layer_weights(cfg, l)
            if keep_inputs:
                kept_layers.append(lw)
            yield lw

    enc = B.EpdEncoder(cfg, gw, layer_stream(), max_tokens=T, max_segments=len(cu) - 1, max_items=len(grids))
    if gemm_tile != -1 or attn_rows != 0:      # tuning experiments: one kernel variant forced for the whole call
        enc.set_tuning(gemm_tile, attn_rows // 128)
    log("[bench] inputs generated and uploaded in %.1f s; workspace %.2f GB" % (time.perf_counter() - t0, enc.workspace_bytes / 1e9))
    p_dev = B.to_device_patches(patches, cfg.dtype)
    out = torch.empty((Tm, cfg.out_dim), dtype=B.torch_dtype(cfg.dtype), device="cuda:0")

    # ---- warm-up, then one call per step with HIP events around each launch of that step
    for _ in range(max(1, warmup)):
        enc.encode(p_dev, cu, grid, out)
    torch.cuda.synchronize()
    table = {}
    for step in range(B.EPD_STEP_COUNT):
        enc.set_timing(step)
        enc.encode(p_dev, cu, grid, out)
        torch.cuda.synchronize()
        table[B.STEP_NAMES[step]] = enc.get_timing()
    enc.set_timing(-1)
    tot = sum(v[0] for v in table.values())
    log("[bench] per-step kernel time of one call (HIP events around each launch):")
    steps_roof = {}
    for k, (ms, n, work) in table.items():
        if n == 0 or k == "plan":
            continue
        rate = work / (ms * 1e-3) if ms > 0 else 0.0
        hbm = k == "norm"
        peak = PEAK_HBM_GBS if hbm else PEAK_BF16_TFLOPS
        ach = rate / (1e9 if hbm else 1e12)
        steps_roof[k] = {"bound": "hbm" if hbm else "mfma", "achieved": ach, "peak": peak, "unit": "GB/s" if hbm else "TFLOP/s",
                         "frac": ach / peak, "launches": n, "avg_launch_ms": ms / n,
                         ("bytes_per_launch" if hbm else "flops_per_launch"): work / n}
        log("    %-12s %4d launches %9.3f ms  %5.1f%%  %8.1f %s  (%.1f%% of peak)" % (k, n, ms, 100 * ms / tot, ach, steps_roof[k]["unit"], 100 * ach / peak))
    if "merge" in steps_roof:
        # the merger's A operand is a 2x2 gather of the normalised rows: bytes it has to move at least
        # (gathered rows once, weights once, output once) over the kernel's time
        es = 2 if cfg.dtype == "bf16" else 4
        gbytes = (Tm * cfg.merge ** 2 * cfg.hidden + cfg.out_dim * cfg.merge ** 2 * cfg.hidden + Tm * cfg.out_dim) * es
        steps_roof["merge"]["gather_algorithmic_GBs"] = gbytes / (table["merge"][0] * 1e-3) / 1e9
    if "qkv" in steps_roof and cfg.rope != "none":
        # rotary is fused into the QKV epilogue: what it adds to that kernel's memory side is the
        # (cos, sin) table of the call, T x d/2 pairs of 8 bytes, read once per launch algorithmically
        rbytes = T * (cfg.head_dim // 2) * 8
        steps_roof["qkv"]["fused_rotary_table_bytes_per_launch"] = rbytes
        steps_roof["qkv"]["fused_rotary_algorithmic_GBs"] = rbytes / (steps_roof["qkv"]["avg_launch_ms"] * 1e-3) / 1e9
    mat_steps = [k for k in steps_roof if k != "norm"]
    dom = max(mat_steps, key=lambda k: table[k][0])
    dom_id = B.STEP_NAMES.index(dom)

    # ---- timed region: exactly `steps` calls; the dominant kernel is bracketed by HIP events.
    # in_flight N > 1: N encoders (own workspace and output each) on N streams of default priority
    # take the steps in turn, so that kernels of different batches fill each other's idle compute
    # units; the default, 1, is the plain sequence of calls on one stream
    extra = []
    if in_flight > 1:
        for _ in range(in_flight - 1):
            extra.append((B.EpdEncoder(cfg, gw, (layer0 if l == 0 else W.layer_weights(cfg, l) for l in range(cfg.num_layers)),
                                       max_tokens=T, max_segments=len(cu) - 1, max_items=len(grids)),
                          torch.empty_like(out), torch.cuda.Stream()))
        for e, o, st in extra:
            with torch.cuda.stream(st):
                e.encode(p_dev, cu, grid, o)
        torch.cuda.synchronize()
    lanes = [(enc, out, torch.cuda.Stream() if extra else torch.cuda.current_stream())] + extra
    enc.set_timing(dom_id)
    torch.cuda.synchronize()
    with PowerSampler() as power:
        t0 = time.perf_counter()
        for i in range(steps):
            e, o, st = lanes[i % len(lanes)]
            with torch.cuda.stream(st):
                e.encode(p_dev, cu, grid, o)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    dom_ms, dom_n, dom_work = enc.get_timing()
    enc.set_timing(-1)
    if extra:
        assert all(torch.equal(o, out) for _, o, _ in extra), "batches in flight disagree"
        for e, _, _ in extra:
            e.close()

    ms_per_step = dt / steps * 1e3
    fl, fl_attn = flops_per_call(cfg, T, Tm, cu)
    tfl = fl / (ms_per_step * 1e-3) / 1e12
    achieved = dom_work / (dom_ms * 1e-3) / 1e12
    log("[bench] %s: %.3f ms/step, %.0f visual tokens/s, %.1f TFLOP/s end to end (%.1f%% of bf16 peak); dominant kernel %s at %.1f TFLOP/s"
        % (cfg.name, ms_per_step, Tm * steps / dt, tfl, 100 * tfl / PEAK_BF16_TFLOPS, dom, achieved))
    if power.summary():
        log("[bench] board power during the timed steps: mean %.0f W, max %.0f W, limit %.0f W" % (power.summary()["mean_w"], power.summary()["max_w"], power.summary()["cap_w"] or 0))
    traffic, traffic_src = (None, "depth, segments, data or kernel variants differ from the profiled run") if (layers_override is not None or segments != "item" or in_flight != 1 or zero_data or gemm_tile != -1 or attn_rows != 0) \
        else stored_traffic(name, dom)
    res = {
        "name": name, "cfg": cfg, "grids": grids, "cu": cu, "grid": grid, "T": T, "Tm": Tm,
        "value": Tm * steps / dt, "ms_per_step": ms_per_step, "seconds": dt, "tflops": tfl, "flops_per_call": fl,
        "attention_flop_share": fl_attn / fl,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_src,
                     "launches": dom_n, "avg_launch_ms": dom_ms / max(dom_n, 1), "flops_per_launch": dom_work / max(dom_n, 1)},
        "rooflines_per_step": steps_roof,
        "board_power": power.summary(),
        "steps_ms": {k: v[0] for k, v in table.items() if v[1] > 0},
        "workload": "%s: %d layers, D=%d, %dx%d heads, MLP %d, patch %d x temporal %d, %d items, %d attention segments, %d patch tokens -> %d visual tokens"
                    % (cfg.name, cfg.num_layers, cfg.hidden, cfg.num_heads, cfg.head_dim, cfg.mlp_dim, cfg.patch, cfg.temporal_patch,
                       len(grids), len(cu) - 1, T, Tm),
        "enc": enc, "p_dev": p_dev, "out": out, "gw": gw, "layer0": layer0, "layers": kept_layers, "patches": patches,
    }
    return res


def release(res):
    import torch
    res["enc"].close()
    for k in ("enc", "p_dev", "out", "gw", "layer0", "layers", "patches"):
        res.pop(k, None)
    gc.collect()
    torch.cuda.empty_cache()


def summary_block(res):
    return {"workload": res["workload"], "value": res["value"], "unit": "visual tokens/s", "ms_per_step": res["ms_per_step"],
            "patch_tokens_per_s": res["T"] / (res["ms_per_step"] * 1e-3), "tflops_end_to_end": res["tflops"],
            "mfma_util_pct_end_to_end": 100 * res["tflops"] / PEAK_BF16_TFLOPS, "attention_flop_share": res["attention_flop_share"],
            "roofline": res["roofline"], "rooflines_per_step": res["rooflines_per_step"], "steps_ms": res["steps_ms"],
            "board_power": res["board_power"]}


def preprocess_and_store(res, with_store):
    """The step in front of the path (raw uint8 pixels -> packed patch rows) and the one behind it
    (feature store), timed on their own: neither is part of `value`, whose inputs are the packed
    rows already in HBM."""
    import torch
    from paper_2601_11590_amd import binding as B, workloads as W
    cfg, grids, enc, p_dev, out = res["cfg"], res["grids"], res["enc"], res["p_dev"], res["out"]
    if cfg.patch % 2:
        return None, None
    src = [(int(h) * cfg.patch, int(w) * cfg.patch) for _, h, w in grids]
    px = torch.from_numpy(np.concatenate([W.item_pixels_u8(cfg, i, g, s).ravel() for i, (g, s) in enumerate(zip(grids, src))])).to("cuda:0")
    rows = torch.empty_like(p_dev)
    mean, std = [0.5] * cfg.in_channels, [0.25] * cfg.in_channels
    for _ in range(3):
        enc.preprocess(px, src, grids, mean, std, out=rows)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 50
    # a few milliseconds of unrelated GPU work go first, so that the host has queued all the
    # launches by the time the first one runs and the events bracket kernel time only
    blocker = torch.ones((8192, 8192), dtype=torch.bfloat16, device="cuda:0")
    torch.cuda.synchronize()
    for _ in range(8):
        blocker @ blocker
    e0.record()
    for _ in range(reps):
        enc.preprocess(px, src, grids, mean, std, out=rows)
    e1.record()
    torch.cuda.synchronize()
    del blocker
    p_ms = e0.elapsed_time(e1) / reps
    p_bytes = px.numel() + rows.numel() * rows.element_size()
    prep = {"ms": p_ms, "bytes": p_bytes, "achieved_GBs": p_bytes / (p_ms * 1e-3) / 1e9, "peak_GBs": PEAK_HBM_GBS,
            "frac": p_bytes / (p_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "bound": "hbm",
            "note": "epd_preprocess, sources at grid size (no resize); mean of %d launches queued back to back" % reps}
    log("[bench] epd_preprocess: %.4f ms per call, %.1f MB -> %.0f GB/s" % (p_ms, p_bytes / 1e6, prep["achieved_GBs"]))
    store_res = None
    if with_store:
        store = B.MMStore((1 << 20) + 2 * out.numel() * out.element_size())
        offs = np.concatenate([[0], np.cumsum([cfg.in_channels * t * cfg.temporal_patch * hs * ws
                                               for (t, _, _), (hs, ws) in zip(grids, src)])]).astype(np.uint64)
        for _ in range(2):
            store.hash(px, offs, [1] * len(grids))
        t0 = time.perf_counter()
        for _ in range(20):
            store.hash(px, offs, [1] * len(grids))
        h_ms = (time.perf_counter() - t0) / 20 * 1e3           # includes the wait for the keys
        t0 = time.perf_counter()
        _, hit_a, _ = enc.encode_cached(store, 7, px, src, grids, mean, std)
        torch.cuda.synchronize()
        miss_ms = (time.perf_counter() - t0) * 1e3
        t0 = time.perf_counter()
        for _ in range(10):
            _, hit_b, _ = enc.encode_cached(store, 7, px, src, grids, mean, std)
        torch.cuda.synchronize()
        hit_ms = (time.perf_counter() - t0) / 10 * 1e3
        assert not hit_a.any() and hit_b.all()
        store_res = {"hash_ms_per_call_incl_sync": h_ms, "hash_bytes": int(px.numel()),
                     "all_miss_call_ms": miss_ms, "all_hit_call_ms": hit_ms,
                     "note": "epd_store_hash of the items (one launch pair + key copy + wait); "
                             "epd_encode_cached on raw pixels: first call (preprocess + encode + file) vs repeated call"}
        log("[bench] mm store: hash %.3f ms per call (%.1f MB, waits for the keys); encode_cached all-miss %.3f ms, all-hit %.3f ms"
            % (h_ms, px.numel() / 1e6, miss_ms, hit_ms))
        store.close()
    return prep, store_res


def colocation(splits):
    """Operator-level co-location (paper section 3.5, "Physical Co-Location and Spatial
    Multiplexing": stages with dissimilar resource demands disturb each other least).  The
    encoder (C2 batch: matrix cores + exp) runs on a stream restricted by a CU mask to `a` of the
    256 compute units while a neighbour runs on a stream restricted to the other 256 - a: either a
    synthetic memory-bound kernel (epd_probe_stream_read over 2 GiB: a decode-like streaming read)
    or a second encoder.  Every entry is time beside the neighbour / time alone ON THE SAME MASK, so
    what is measured is interference through what the two still share (HBM, the caches behind the
    CUs, power), not the loss of compute units.  Prints one JSON line."""
    import ctypes as C
    import torch
    from paper_2601_11590_amd import binding as B, workloads as W
    hip = C.CDLL("libamdhip64.so")
    hip.hipExtStreamCreateWithCUMask.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.POINTER(C.c_uint32)]
    hip.hipExtStreamCreateWithCUMask.restype = C.c_int
    ncu = torch.cuda.get_device_properties(0).multi_processor_count
    words = (ncu + 31) // 32

    def masked_stream(lo, hi):
        """Stream whose kernels may only use logical compute units [lo, hi).  The driver deals the
        logical units of the mask out to the eight XCDs in turn, so a contiguous range takes the same
        share of every XCD."""
        bits = (C.c_uint32 * words)()
        for cu in range(lo, hi):
            bits[cu // 32] |= 1 << (cu % 32)
        h = C.c_void_p()
        rc = hip.hipExtStreamCreateWithCUMask(C.byref(h), words, bits)
        assert rc == 0 and h.value, "hipExtStreamCreateWithCUMask failed (%d)" % rc
        return torch.cuda.ExternalStream(h.value)

    cfg = W.C2
    grids = W.grids_for(cfg)
    T, Tm = W.num_tokens(grids), W.num_merged_tokens(grids, cfg.merge)
    gw = W.global_weights(cfg)
    layers = [W.layer_weights(cfg, l) for l in range(cfg.num_layers)]
    patches = B.to_device_patches(W.packed_patches(cfg, grids), cfg.dtype)
    cu, grid = W.metadata(grids)
    encs = [B.EpdEncoder(cfg, gw, layers, max_tokens=T, max_segments=len(grids), max_items=len(grids)) for _ in range(2)]
    outs = [torch.empty((Tm, cfg.out_dim), dtype=torch.bfloat16, device="cuda:0") for _ in range(2)]
    nbytes = 2 << 30
    bufs = [torch.ones(nbytes // 4, dtype=torch.int32, device="cuda:0") for _ in range(2)]
    sums = [torch.zeros(65536, dtype=torch.float32, device="cuda:0") for _ in range(2)]

    def op_encode(slot, stream, n_cu):
        encs[slot].set_compute_units(0 if n_cu >= 256 else n_cu)     # the launcher cannot see the stream's mask
        encs[slot].encode(patches, cu, grid, outs[slot])

    def op_read(slot, stream, n_cu):
        B.epd_probe_stream_read(bufs[slot].data_ptr(), nbytes, sums[slot].data_ptr(), 16 * n_cu, stream.cuda_stream)

    ops = {"encode": (op_encode, 6), "read": (op_read, 12)}

    def timed(a, sa, na, b=None, sb=None, nb=0, b_reps=0):
        """ms per launch of op `a` on stream sa, optionally while op `b` keeps stream sb busy."""
        fa, reps = ops[a]
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if b is not None:
            with torch.cuda.stream(sb):
                for _ in range(b_reps):
                    ops[b][0](1, sb, nb)
        with torch.cuda.stream(sa):
            fa(0, sa, na)
            e0.record()
            for _ in range(reps):
                fa(0, sa, na)
            e1.record()
        e1.synchronize()
        ms = e0.elapsed_time(e1) / reps
        torch.cuda.synchronize()
        return ms

    full = masked_stream(0, ncu)
    ref = {k: timed(k, full, ncu) for k in ops}
    log("[colocation] all %d CUs: encode %.3f ms per C2 call, read %.3f ms per 2 GiB (%.0f GB/s)" % (ncu, ref["encode"], ref["read"], nbytes / ref["read"] / 1e6))
    rows = []
    for a_cus in splits:
        sa, sb = masked_stream(0, a_cus), masked_stream(a_cus, ncu)
        nb = ncu - a_cus
        alone = {("encode", "A"): timed("encode", sa, a_cus), ("read", "A"): timed("read", sa, a_cus),
                 ("encode", "B"): timed("encode", sb, nb), ("read", "B"): timed("read", sb, nb)}
        row = {"cus_measured": a_cus, "cus_neighbour": nb,
               "encode_alone_ms": alone["encode", "A"], "read_alone_GBs_on_neighbour_cus": nbytes / alone["read", "B"] / 1e6}
        for a in ops:
            for b in ops:
                # the neighbour's queue lasts several times longer than the measured run
                need = 4.0 * alone[a, "A"] * (ops[a][1] + 1)
                b_reps = int(need / alone[b, "B"]) + 2
                row["%s_beside_%s" % (a, b)] = timed(a, sa, a_cus, b, sb, nb, b_reps) / alone[a, "A"]
        # and the other way round for the mixed pair: the reader on the small mask beside the encoder
        need = 4.0 * alone["read", "B"] * (ops["read"][1] + 1)
        row["read_on_neighbour_cus_beside_encode"] = timed("read", sb, nb, "encode", sa, a_cus, int(need / alone["encode", "A"]) + 2) / alone["read", "B"]
        rows.append(row)
        log("[colocation] encoder on %3d CUs (%.3f ms alone), neighbour on %3d: encode beside read x%.2f, beside encode x%.2f | "
            "read beside read x%.2f, beside encode x%.2f | read on the %d CUs (%.0f GB/s alone) beside the encoder x%.2f"
            % (a_cus, alone["encode", "A"], nb, row["encode_beside_read"], row["encode_beside_encode"], row["read_beside_read"],
               row["read_beside_encode"], nb, nbytes / alone["read", "B"] / 1e6, row["read_on_neighbour_cus_beside_encode"]))
    print(json.dumps({"experiment": "operator co-location on CU-masked streams: time beside the neighbour / time alone on the same mask, one MI355X",
                      "all_cus": {"encode_ms": ref["encode"], "read_ms": ref["read"], "read_GBs": nbytes / ref["read"] / 1e6},
                      "splits": rows}), flush=True)
    for e in encs:
        e.close()


def mfma_peak():
    """Practical ceiling of the bf16 matrix pipes (epd_probe_mfma_rate: register-resident operands,
    no memory traffic) for both instruction shapes, on random and on all-zero operands.  Prints one
    JSON line."""
    import torch
    from paper_2601_11590_amd import binding as B
    out = torch.zeros(256 * 512, dtype=torch.float32, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    res, watts = {}, {}
    for shape, sname in ((0, "v_mfma_f32_32x32x16_bf16"), (1, "v_mfma_f32_16x16x32_bf16")):
        for zero in (False, True):
            B.epd_probe_mfma_rate(shape, zero, 200, out.data_ptr(), st)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 300       # 6 - 8 s per case: the power sensor settles within the first second
            with PowerSampler() as power:
                e0.record()
                for _ in range(reps):
                    fl = B.epd_probe_mfma_rate(shape, zero, 20000, out.data_ptr(), st)
                e1.record()
                torch.cuda.synchronize()
            tf = reps * fl / (e0.elapsed_time(e1) * 1e-3) / 1e12
            pw = power.summary(tail=0.75)
            key = "%s, %s operands" % (sname, "all-zero" if zero else "random")
            res[key] = tf
            watts[key] = pw
            log("[mfma-peak] %-28s %-8s operands: %7.1f TFLOP/s (%.1f%% of %.0f)%s" % (sname, "all-zero" if zero else "random", tf, 100 * tf / PEAK_BF16_TFLOPS, PEAK_BF16_TFLOPS,
                                                                                       "  board power %.0f W of %.0f" % (pw["mean_w"], pw["cap_w"] or 0) if pw else ""))
    print(json.dumps({"experiment": "bf16 matrix-core rate on register-resident operands, 2 waves per SIMD on all 256 CUs, TFLOP/s",
                      "published_peak": PEAK_BF16_TFLOPS, "measured": res, "board_power": watts}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C5", help="headline workload: C5 (default, the largest single-GPU configuration) | C2 | C3 | C4 | "
                         "T42 (the six image resolutions of the paper's Table 4_2 as one batch)")
    ap.add_argument("--others", default=None,
                    help="comma-separated configurations timed briefly beside the headline (default: C2,C3,C4,T42 with C5, none otherwise; '' = none)")
    ap.add_argument("--layers", type=int, default=None, help="override depth (experiments only; never the headline)")
    ap.add_argument("--segments", default="item", choices=["item", "frame"],
                    help="attention segments: one per image / clip (default) or one per video frame (windowed attention)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--gemm-tile", type=int, default=-1, choices=[-1, 0, 2, 4, 5],
                    help="tuning experiment: force one bf16 GEMM tile for every GEMM of the call (0 = 256x256, 2 = 256x128, 4 = 128x128, "
                         "5 = 320x256; -1 = the library's plan); never the headline")
    ap.add_argument("--attn-rows", type=int, default=0, choices=[0, 128, 256],
                    help="tuning experiment: force the attention kernel's query rows per block (0 = the library's choice)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy 5 times (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--in-flight", type=int, default=1,
                    help="batches in flight on separate streams (serving mode; default 1 = one stream)")
    ap.add_argument("--zero-data", action="store_true",
                    help="experiment: all weights and inputs zero (same kernels, no operand toggling): the pipeline-bound rate "
                         "beside the power-bound rate of the default run; never the headline")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="only measure the matrix-core rate on register-resident operands (random and all-zero)")
    ap.add_argument("--colocation", default=None, metavar="CUS[,CUS...]",
                    help="only run the co-location experiment (section 3.5): compute units given to the encoder's stream, "
                         "e.g. 224,192,128; the neighbour's stream gets the others")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
            "--gpus %d is not supported. Items would shard across GPUs by image with replicated "
            "weights; nothing here launches more than one rank." % args.gpus)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.colocation:
        colocation([int(v) for v in args.colocation.split(",")])
        return
    if args.mfma_peak:
        mfma_peak()
        return
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("[bench] copied 5 x 1 GiB (reads 1 GiB and writes 1 GiB per launch)")
        return

    plain = args.layers is None and args.segments == "item" and args.in_flight == 1 and not args.zero_data and args.gemm_tile == -1 and args.attn_rows == 0
    small = args.config in ("C2", "C3")           # the oracle runs these at full depth in seconds
    head = measure(args.config, args.steps, args.warmup, args.in_flight, args.layers, args.segments,
                   keep_inputs=small and not args.no_cpu and not args.zero_data, zero_data=args.zero_data,
                   gemm_tile=args.gemm_tile, attn_rows=args.attn_rows)
    prep, store_res = preprocess_and_store(head, with_store=args.config == "C2" and plain)
    gpu_out = head["out"].float().cpu().numpy()
    stored = stored_rows_parity(args.config, gpu_out) if plain else None
    cpu = None
    if not args.no_cpu and not args.zero_data:
        if small:
            n = len(head["grids"]) if args.config == "C2" else 3
            cpu = cpu_baseline_full(head["cfg"], head["gw"], head["layers"], head["patches"], head["grid"], gpu_out, n) if args.segments == "item" else None
        elif head["cfg"].num_layers > 0:
            cpu = cpu_baseline_depth_sample(head["cfg"], head["gw"], head["layer0"], head["patches"], head["grid"])
    cfg = head["cfg"]
    line = {
        "metric": "visual tokens/sec (ViT encode fwd, 1 GPU) + MFMA util % of bf16 peak",
        "value": head["value"], "unit": "visual tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "batches_in_flight": args.in_flight, "forced_gemm_tile": args.gemm_tile, "forced_attn_rows": args.attn_rows, "patch_tokens": head["T"], "visual_tokens": head["Tm"],
                   "patch_tokens_per_s": head["T"] / (head["ms_per_step"] * 1e-3), "tflops_end_to_end": head["tflops"],
                   "mfma_util_pct_end_to_end": 100 * head["tflops"] / PEAK_BF16_TFLOPS,
                   "attention_flop_share": head["attention_flop_share"]},
        "roofline": head["roofline"],
        "rooflines_per_step": head["rooflines_per_step"],
        "cpu_baseline": cpu,
        "parity_vs_stored_oracle_rows": stored,
        "preprocess": prep,
        "mm_store": store_res,
        "steps_ms": head["steps_ms"],
        "board_power": head["board_power"],
        "peaks": {"bf16_mfma_TFLOPs": PEAK_BF16_TFLOPS, "hbm_GBs": PEAK_HBM_GBS},
    }
    release(head)
    others = args.others
    if others is None:
        others = "C2,C3,C4,T42" if (args.config == "C5" and plain) else ""
    blocks = {}
    for name in [n for n in others.split(",") if n]:
        r = measure(name, 3 if name == "T42" else 5, 1 if name == "T42" else 2)
        blocks[name] = summary_block(r)
        if name in ("C4",):
            blocks[name]["parity_vs_stored_oracle_rows"] = stored_rows_parity(name, r["out"].float().cpu().numpy())
        release(r)
    line["others"] = blocks
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
