#!/usr/bin/env python3
"""Throughput of the Encode stage (ViT forward, V_m = E(I_m); paper section 3.1, Eq. 1) on one
MI355X: visual tokens per second on the 24-layer bf16 encoder with a batch of 8 images of
448 x 448 (6272 packed patch tokens -> 1568 visual tokens), synthetic seeded inputs.

One "step" is one epd_encode call: plan, patch embedding, 24 transformer blocks, final norm,
2x2 merge and projection, with the packed patches and weights already resident in HBM.

Prints ONE JSON line on stdout; progress and the per-step table go to stderr.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(cfg, gw, layers, patches, cu, grid, gpu_out, n_items):
    """Time the CPU oracle, as it stands, on the first n_items images of the same batch."""
    from oracle import vit_encode as O
    from paper_2601_11590_amd import workloads as W
    grids = [tuple(int(v) for v in g) for g in grid[:n_items]]
    T = W.num_tokens(grids)
    Tm = W.num_merged_tokens(grids, cfg.merge)
    cu1, g1 = W.metadata(grids)
    t0 = time.perf_counter()
    ref = O.encode(cfg, gw, layers, patches[:T], cu1, g1)
    dt = time.perf_counter() - t0
    got = gpu_out[:Tm].astype(np.float64)
    cos = (got * ref).sum(-1) / (np.linalg.norm(got, axis=-1) * np.linalg.norm(ref, axis=-1))
    rel = np.abs(got - ref).max(-1) / np.abs(ref).max(-1)
    log("[bench] oracle on %d image(s): %.2f s; GPU rows vs oracle: min cos %.6f, max rel %.3e"
        % (n_items, dt, cos.min(), rel.max()))
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env))
    return {"value": Tm / dt, "unit": "visual tokens/s", "cores": cores, "kind": "oracle",
            "sample": "first %d of the 8 images (%d patch tokens -> %d visual tokens), all %d layers, "
                      "fp64 NumPy, one run" % (n_items, T, Tm, cfg.num_layers),
            "seconds": dt, "parity_min_cos": float(cos.min()), "parity_max_rel": float(rel.max())}


def colocation():
    """Operator-level co-location (paper section 3.5, "Physical Co-Location and Spatial Multiplexing"):
    how much one kind of work slows down when another kind runs beside it on the same GPU, for work
    bound by different units.  Rows = the measured operator, columns = the neighbour; entries =
    time beside the neighbour / time alone.  Prints one JSON line."""
    import torch
    from paper_2601_11590_amd import binding as B, workloads as W
    cfg = W.C2
    grids = W.grids_for(cfg)
    T, Tm = W.num_tokens(grids), W.num_merged_tokens(grids, cfg.merge)
    gw = W.global_weights(cfg)
    layers = [W.layer_weights(cfg, l) for l in range(cfg.num_layers)]
    patches = B.to_device_patches(W.packed_patches(cfg, grids), cfg.dtype)
    cu, grid = W.metadata(grids)
    encs = [B.EpdEncoder(cfg, gw, layers, max_tokens=T, max_segments=len(grids), max_items=len(grids)) for _ in range(2)]
    outs = [torch.empty((Tm, cfg.out_dim), dtype=torch.bfloat16, device="cuda:0") for _ in range(2)]
    src = [torch.ones(1 << 27, dtype=torch.float32, device="cuda:0") for _ in range(2)]     # 512 MiB each
    dst = [torch.empty_like(x) for x in src]
    stores = [B.MMStore(2 << 20) for _ in range(2)]
    blob = [torch.randint(0, 256, (64 << 20,), dtype=torch.uint8, device="cuda:0") for _ in range(2)]
    nrm = [torch.randn((1 << 16, 1024), dtype=torch.float32, device="cuda:0") for _ in range(2)]

    # one unit of each kind of work, on the current stream; slot 0 = measured, 1 = neighbour
    ops = {
        "encode (matrix cores + exp)": lambda i: encs[i].encode(patches, cu, grid, outs[i]),
        "copy 512 MiB (HBM)": lambda i: dst[i].copy_(src[i]),
        "hash 64 MiB (integer ALU)": lambda i: stores[i].hash(blob[i], [0, blob[i].numel()], [1]),
        "softmax 64k x 1024 fp32 (HBM + exp)": lambda i: torch.softmax(nrm[i], dim=-1),
    }
    # the hash call waits for its keys (it is synchronous by contract), so it cannot sit in a queue
    # beside something else: it is measured, never a neighbour
    names = list(ops)
    neighbours = [n for n in names if not n.startswith("hash")]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    reps = {"encode (matrix cores + exp)": 6, "copy 512 MiB (HBM)": 60, "hash 64 MiB (integer ALU)": 20,
            "softmax 64k x 1024 fp32 (HBM + exp)": 60}

    def timed(a, b):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        if b is not None:
            with torch.cuda.stream(s2):
                for _ in range(reps[b] * 6):          # a queue several times longer than the measured run
                    ops[b](1)
        with torch.cuda.stream(s1):
            ops[a](0)
            e0.record()
            for _ in range(reps[a]):
                ops[a](0)
            e1.record()
        e1.synchronize()
        ms = e0.elapsed_time(e1) / reps[a]
        torch.cuda.synchronize()
        return ms

    alone = {a: min(timed(a, None) for _ in range(2)) for a in names}
    table = {a: {b: timed(a, b) / alone[a] for b in neighbours} for a in names}
    for a in names:
        log("[colocation] %-38s alone %8.3f ms | " % (a, alone[a]) + "  ".join("beside %s: x%.2f" % (b.split(" (")[0], table[a][b]) for b in neighbours))
    print(json.dumps({"experiment": "operator co-location slowdown (time beside neighbour / time alone), one MI355X, two streams of default priority",
                      "alone_ms": alone, "slowdown": table}), flush=True)
    for e in encs:
        e.close()
    for st in stores:
        st.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C2", help="C2 (headline) | C3 | C4 | C5 (other single-GPU shapes)")
    ap.add_argument("--layers", type=int, default=None, help="override depth (non-headline experiments only)")
    ap.add_argument("--cpu-items", type=int, default=8, help="images of the batch the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy 5 times (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--in-flight", type=int, default=1,
                    help="batches in flight on separate streams (serving mode; default 1 = one stream)")
    ap.add_argument("--colocation", action="store_true",
                    help="only run the operator co-location experiment (section 3.5) and print its table")
    args = ap.parse_args()
    if args.colocation:
        if args.gpus != 1:
            log("bench.py: one GPU only"); sys.exit(2)
        colocation()
        return
    if args.copy_calibration:
        import torch
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        log("[bench] copied 5 x 1 GiB (reads 1 GiB and writes 1 GiB per launch)")
        return
    if args.gpus != 1:
        log("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
            "--gpus %d is not supported. Items would shard across GPUs by image with replicated "
            "weights; nothing here launches more than one rank." % args.gpus)
        sys.exit(2)

    import torch
    from paper_2601_11590_amd import binding as B, workloads as W

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    cfg = W.CONFIGS[args.config]
    grids = W.grids_for(cfg)
    if args.layers is not None:
        cfg = cfg.replace(num_layers=args.layers)
    T, Tm = W.num_tokens(grids), W.num_merged_tokens(grids, cfg.merge)
    log("[bench] %s: %d items, T=%d patch tokens -> %d visual tokens, L=%d" % (cfg.name, len(grids), T, Tm, cfg.num_layers))

    t0 = time.perf_counter()
    gw = W.global_weights(cfg)
    layers = [W.layer_weights(cfg, l) for l in range(cfg.num_layers)]
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids)
    log("[bench] inputs generated in %.1f s" % (time.perf_counter() - t0))

    enc = B.EpdEncoder(cfg, gw, layers, max_tokens=T, max_segments=len(cu) - 1, max_items=len(grids))
    p_dev = B.to_device_patches(patches, cfg.dtype)
    out = torch.empty((Tm, cfg.out_dim), dtype=B.torch_dtype(cfg.dtype), device="cuda:0")
    log("[bench] workspace %.2f GB" % (enc.workspace_bytes / 1e9))

    # ---- warm-up, with a per-step timing pass to find the dominant kernel
    for _ in range(max(1, args.warmup)):
        enc.encode(p_dev, cu, grid, out)
    torch.cuda.synchronize()
    table = {}
    for step in range(B.EPD_STEP_COUNT):
        enc.set_timing(step)
        enc.encode(p_dev, cu, grid, out)
        torch.cuda.synchronize()
        ms, n, work = enc.get_timing()
        table[B.STEP_NAMES[step]] = (ms, n, work)
    enc.set_timing(-1)
    tot = sum(v[0] for v in table.values())
    log("[bench] per-step kernel time of one call (HIP events around each launch):")
    for k, (ms, n, work) in table.items():
        if n == 0:
            continue
        rate = work / (ms * 1e-3) if ms > 0 else 0.0
        unit = "GB/s" if k == "norm" else "TFLOP/s"
        scale = 1e9 if k == "norm" else 1e12
        log("    %-12s %4d launches %9.3f ms  %5.1f%%  %8.1f %s" % (k, n, ms, 100 * ms / tot, rate / scale, unit))
    mat_steps = [k for k in table if k not in ("plan", "norm") and table[k][1] > 0]
    dom = max(mat_steps, key=lambda k: table[k][0])
    dom_id = B.STEP_NAMES.index(dom)

    # ---- timed region: exactly K steps; the dominant kernel is bracketed by HIP events
    # --in-flight N > 1: N encoders (own workspace and output each) on N streams of default
    # priority take the steps in turn, so that kernels of different batches fill each other's
    # idle compute units; the default, 1, is the plain sequence of calls on one stream
    extra = []
    if args.in_flight > 1:
        for _ in range(args.in_flight - 1):
            extra.append((B.EpdEncoder(cfg, gw, layers, max_tokens=T, max_segments=len(cu) - 1, max_items=len(grids)),
                          torch.empty_like(out), torch.cuda.Stream()))
        for e, o, st in extra:
            with torch.cuda.stream(st):
                e.encode(p_dev, cu, grid, o)
        torch.cuda.synchronize()
    # with several lanes none of them is the default stream (whose launches order against the others')
    lanes = [(enc, out, torch.cuda.Stream() if extra else torch.cuda.current_stream())] + extra
    enc.set_timing(dom_id)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
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

    ms_per_step = dt / args.steps * 1e3
    value = Tm * args.steps / dt
    achieved = dom_work / (dom_ms * 1e-3) / 1e12          # TFLOP/s over the kernel's own time
    D, F, L = cfg.hidden, cfg.mlp_dim, cfg.num_layers
    flops_call = (2.0 * T * cfg.patch_dim * D + L * (8.0 * T * D * D + 4.0 * T * D * F)
                  + L * sum(4.0 * float(cu[i + 1] - cu[i]) ** 2 * D for i in range(len(cu) - 1))
                  + 2.0 * Tm * (cfg.merge ** 2 * D) * cfg.out_dim)
    log("[bench] %.3f ms/step, %.0f visual tokens/s, %.1f TFLOP/s end to end (%.1f%% of bf16 peak)"
        % (ms_per_step, value, flops_call / (ms_per_step * 1e-3) / 1e12,
           100 * flops_call / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS))

    # ---- the step in front of the path (raw uint8 pixels -> packed patch rows), timed on its
    # own: it is not part of `value`, whose inputs are the packed rows already in HBM
    prep = None
    store_res = None
    if cfg.patch % 2 == 0:
        src = [(int(h) * cfg.patch, int(w) * cfg.patch) for _, h, w in grids]
        px = torch.from_numpy(np.concatenate([W.item_pixels_u8(cfg, i, g, s).ravel()
                                              for i, (g, s) in enumerate(zip(grids, src))])).to("cuda:0")
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
        # ---- the step behind it: the feature store (hash of the input as key; a hit skips the encoder)
        if args.config == "C2" and args.layers is None:
            store = B.MMStore((1 << 20) + 2 * out.numel() * out.element_size())
            offs = np.concatenate([[0], np.cumsum([cfg.in_channels * t * cfg.temporal_patch * hs * ws
                                                   for (t, _, _), (hs, ws) in zip(grids, src)])]).astype(np.uint64)
            for _ in range(2):
                store.hash(px, offs, [1] * len(grids))
            t0 = time.perf_counter()
            for _ in range(20):
                store.hash(px, offs, [1] * len(grids))
            h_ms = (time.perf_counter() - t0) / 20 * 1e3           # includes the wait for the 128 bytes of keys
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
                         "note": "epd_store_hash of the 8 images (one launch pair + key copy + wait); "
                                 "epd_encode_cached on raw pixels: first call (preprocess + encode + file) vs repeated call"}
            log("[bench] mm store: hash %.3f ms per call (%.1f MB, waits for the keys); encode_cached all-miss %.3f ms, all-hit %.3f ms"
                % (h_ms, px.numel() / 1e6, miss_ms, hit_ms))
            store.close()
        del px, rows

    gpu_out = out.float().cpu().numpy()
    cpu = None
    if args.cpu_items > 0:
        cpu = cpu_baseline(cfg, gw, layers, patches, cu, grid, gpu_out, min(args.cpu_items, len(grids)))

    # HBM-side bytes per launch of the dominant kernel come from rocprofv3 --pmc FETCH_SIZE /
    # WRITE_SIZE runs of this same command (see profiles/); they cannot be collected in-process.
    traffic = None
    tfile = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "c2_bench_hbm_traffic.txt")
    if args.config == "C2" and args.layers is None and os.path.exists(tfile):
        for line in open(tfile):
            parts = line.split()
            if len(parts) >= 3 and parts[0] == "TRAFFIC_BYTES_PER_LAUNCH" and parts[1] == dom:
                traffic = float(parts[2])
    res = {
        "metric": "visual tokens/sec (ViT encode fwd, 1 GPU) + MFMA util % of bf16 peak",
        "value": value, "unit": "visual tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "%s: %d layers, D=%d, %dx%d heads, MLP %d, patch %d, %d items, %d patch tokens -> %d visual tokens"
                               % (cfg.name, L, D, cfg.num_heads, cfg.head_dim, F, cfg.patch, len(grids), T, Tm),
                   "batches_in_flight": args.in_flight, "patch_tokens": T, "visual_tokens": Tm, "patch_tokens_per_s": T * args.steps / dt,
                   "tflops_end_to_end": flops_call / (ms_per_step * 1e-3) / 1e12,
                   "mfma_util_pct_end_to_end": 100 * flops_call / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "launches": dom_n, "avg_launch_ms": dom_ms / max(dom_n, 1),
                     "flops_per_launch": dom_work / max(dom_n, 1)},
        "cpu_baseline": cpu,
        "preprocess": prep,
        "mm_store": store_res,
        "steps_ms": {k: v[0] for k, v in table.items() if v[1] > 0},
    }
    enc.close()
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
