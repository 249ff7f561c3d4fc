"""Full-depth parity of the two largest benchmark configurations: C4 (27 layers, one 28 224-token
sequence, head dim 72) and C5 (45 layers, four 8192-token video clips, head dim 128) run once
through the C ABI exactly as bench.py launches them, and the sampled output rows are compared
with the fp64 oracle's rows stored under tests/golden/ (written on the CPU by
tests/golden/make_full_depth_rows.py, which calls nothing but oracle/ and the input generators;
the oracle needs tens of minutes per configuration, so it is not run inside the test).
Tolerances as everywhere: per-token cosine >= 0.999, max-norm relative error <= 2e-2."""

import os

import numpy as np
import pytest

from paper_2601_11590_amd import workloads as W
from parity_util import check, log

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def run_full(cfg):
    import torch
    from paper_2601_11590_amd import binding as B
    grids = W.grids_for(cfg)
    gw = W.global_weights(cfg)
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids)
    # layers are drawn one at a time by the encoder's constructor: 45 layers of C5 are 22 GB as float32
    enc = B.EpdEncoder(cfg, gw, (W.layer_weights(cfg, l) for l in range(cfg.num_layers)), max_tokens=patches.shape[0],
                       max_segments=len(grids), max_items=len(grids))
    try:
        got = enc.encode(B.to_device_patches(patches, cfg.dtype), cu, grid)
        torch.cuda.synchronize()
        got = got.float().cpu().numpy()
    finally:
        enc.close()
    return got


@pytest.mark.parametrize("name", ["C4", "C5"])
def test_full_depth_rows_against_stored_oracle_rows(name):
    cfg = W.CONFIGS[name]
    z = np.load(os.path.join(GOLDEN, "%s_full_depth_rows.npz" % name.lower()), allow_pickle=False)
    rows, want, first = z["rows"], z["values"], int(z["first_row_in_batch"])
    log("case %s full depth (%d layers): %d stored oracle rows of a %s part starting at output row %d"
        % (cfg.name, cfg.num_layers, len(rows), tuple(int(v) for v in z["out_shape"]), first))
    got = run_full(cfg)
    assert got.shape == (W.num_merged_tokens(W.grids_for(cfg), cfg.merge), cfg.out_dim) and np.isfinite(got).all()
    assert want.shape == (len(rows), cfg.out_dim) and len(rows) >= 64
    check(cfg, got[first + rows], want, "%d sampled rows, %d layers" % (len(rows), cfg.num_layers))
