"""Helpers shared by the GPU parity tests: run the HIP library and the CPU oracle on the same
seeded inputs and compare with the tolerances the benchmark states."""

import sys

import numpy as np


def log(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def error_metrics(got: np.ndarray, ref: np.ndarray):
    """(max abs error, min per-token cosine, max per-token max-norm relative error)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    diff = np.abs(got - ref)
    num = (got * ref).sum(-1)
    den = np.linalg.norm(got, axis=-1) * np.linalg.norm(ref, axis=-1)
    cos = num / np.maximum(den, 1e-300)
    rel = diff.max(-1) / np.maximum(np.abs(ref).max(-1), 1e-300)
    return float(diff.max()), float(cos.min()), float(rel.max())


# tolerances stated for the benchmark
F32_MAX_ABS = 1e-4
BF16_MIN_COS = 0.999
BF16_MAX_REL = 2e-2


def check(cfg, got, ref, what=""):
    mabs, cos, rel = error_metrics(got, ref)
    log("  %s %s: max_abs=%.3e min_cos=%.6f max_rel=%.3e" % (cfg.name, what, mabs, cos, rel))
    assert np.isfinite(np.asarray(got, np.float64)).all(), "non-finite output"
    if cfg.dtype == "f32":
        assert mabs <= F32_MAX_ABS, (what, mabs)
    else:
        assert cos >= BF16_MIN_COS, (what, cos)
        assert rel <= BF16_MAX_REL, (what, rel)
    return mabs, cos, rel


def run_gpu(cfg, gw, layers, patches, cu, grid, want_hidden=False, max_tokens=None, segments=None, items=None,
            gemm_tile=-1, attn_groups=0):
    """One epd_encode call through the C ABI; returns float64 arrays.  gemm_tile / attn_groups
    force a kernel variant through the library's tuning hook (-1 / 0 = its own choice)."""
    import torch
    from paper_2601_11590_amd import binding as B
    enc = B.EpdEncoder(cfg, gw, layers, max_tokens=max_tokens or int(patches.shape[0]),
                       max_segments=segments or max(1, len(cu) - 1), max_items=items or max(1, len(grid)))
    try:
        if gemm_tile != -1 or attn_groups != 0:
            enc.set_tuning(gemm_tile, attn_groups)
        p = B.to_device_patches(patches, cfg.dtype)
        y = enc.encode(p, cu, grid)
        torch.cuda.synchronize()
        out = y.float().cpu().numpy().astype(np.float64)
        hid = enc.hidden().cpu().numpy().astype(np.float64) if want_hidden else None
        torch.cuda.synchronize()
    finally:
        enc.close()
    return (out, hid) if want_hidden else out
