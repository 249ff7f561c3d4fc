#!/usr/bin/env python3
"""Writes the full-depth expected rows of the two largest benchmark configurations.

CPU only.  Imports nothing but the fp64 oracle (oracle/vit_encode.py) and the seeded input
generators (paper_2601_11590_amd/workloads.py, which holds no arithmetic of the method) and
evaluates V_m = E(I_m) (paper section 3.1, Eq. 1) at the configurations' full depth:

  C4  one 2688 x 2688 image, a single 28 224-token attention segment, 27 layers, head dim 72
      -> 7056 x 3584 visual tokens;
  C5  the LAST of the four 16-frame clips of the video batch alone (block-diagonal attention
      makes its rows in the batch equal to the clip encoded alone), 8192 tokens, 45 layers,
      head dim 128 -> 2048 x 8192 visual tokens.

Of each output the rows `sample_rows(n)` are stored, float64, as
tests/golden/<name>_full_depth_rows.npz (arrays `rows`, `values`), to be read with
numpy.load(..., allow_pickle=False).  The GPU tests run the whole configuration once through
the C ABI and compare exactly these rows.  Each run takes tens of minutes on 8-16 cores.

usage: python tests/golden/make_full_depth_rows.py C4|C5 [--layers N]
"""

import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import vit_encode as O                      # noqa: E402
from paper_2601_11590_amd import workloads as W         # noqa: E402

N_ROWS = 96


def sample_rows(n_out: int, n: int = N_ROWS) -> np.ndarray:
    """First row, last row and an even spread between them (window corners and edges of the
    merged grid fall in naturally because the stride is not a multiple of the grid width)."""
    return np.unique(np.round(np.linspace(0, n_out - 1, n)).astype(np.int64))


def inputs(name: str):
    """(cfg, patches of the part the oracle evaluates, cu_seqlens, grid_thw, first output row
    of that part inside the full batch's output)."""
    cfg = W.CONFIGS[name]
    grids = W.grids_for(cfg)
    if name == "C4":
        part, first = [0], 0
    elif name == "C5":
        part = [len(grids) - 1]
        first = W.num_merged_tokens(grids[:-1], cfg.merge)
    else:
        raise SystemExit("C4 or C5")
    rows = [W.patchify(W.item_pixels(cfg, i, grids[i]), cfg.patch, cfg.temporal_patch) for i in part]
    patches = W.round_to_dtype(np.concatenate(rows, axis=0), cfg.dtype)
    cu, grid = W.metadata([grids[i] for i in part])
    return cfg, patches, cu, grid, first


def main():
    name = sys.argv[1]
    cfg, patches, cu, grid, first = inputs(name)
    if "--layers" in sys.argv:                                   # dry runs only; never stored
        cfg = cfg.replace(num_layers=int(sys.argv[sys.argv.index("--layers") + 1]))
    full = cfg.num_layers == W.CONFIGS[name].num_layers

    def layers():
        for l in range(cfg.num_layers):
            t0 = time.perf_counter()
            lw = W.layer_weights(cfg, l)
            print("[golden %s] layer %d/%d (weights drawn in %.1f s, %.0f s since start)"
                  % (name, l + 1, cfg.num_layers, time.perf_counter() - t0, time.perf_counter() - t_start), flush=True)
            yield lw

    t_start = time.perf_counter()
    y = O.encode(cfg, W.global_weights(cfg), layers(), patches, cu, grid)
    secs = time.perf_counter() - t_start
    rows = sample_rows(y.shape[0])
    print("[golden %s] oracle output %s in %.0f s; storing %d rows" % (name, y.shape, secs, len(rows)), flush=True)
    if not full:
        print("[golden %s] reduced depth: nothing stored" % name)
        return
    out = os.path.join(HERE, "%s_full_depth_rows.npz" % name.lower())
    np.savez(out, rows=rows, values=np.ascontiguousarray(y[rows], dtype=np.float64),
             first_row_in_batch=np.int64(first), out_shape=np.asarray(y.shape, np.int64),
             oracle_seconds=np.float64(secs))
    print("[golden %s] wrote %s" % (name, out))


if __name__ == "__main__":
    main()
