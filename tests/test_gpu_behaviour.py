"""GPU behaviour of the C-ABI library beyond plain parity: determinism, segment isolation,
batch invariance, error handling, handle reuse, and the shapes of the larger configurations
(at reduced depth or sampled against the oracle, which is too slow for them in full)."""

import numpy as np
import pytest

from oracle import vit_encode as O
from paper_2601_11590_amd import workloads as W
from parity_util import check, error_metrics, log

pytestmark = pytest.mark.gpu


def small(dtype, **kw):
    base = dict(name="beh-" + dtype, dtype=dtype, num_layers=2, hidden=256, num_heads=4, head_dim=64,
                mlp_dim=512, patch=4, temporal_patch=1, norm="rmsnorm", rope="2d", rope_pairs=(0, 16, 16),
                out_dim=192, seed=5)
    base.update(kw)
    return W.EncoderConfig(**base)


def make_encoder(cfg, max_tokens, segs=16, items=16):
    from paper_2601_11590_amd import binding as B
    gw, layers = W.all_weights(cfg)
    return B.EpdEncoder(cfg, gw, layers, max_tokens=max_tokens, max_segments=segs, max_items=items), gw, layers


def run(enc, cfg, patches, cu, grid, hidden=False):
    import torch
    from paper_2601_11590_amd import binding as B
    y = enc.encode(B.to_device_patches(patches, cfg.dtype), cu, grid)
    torch.cuda.synchronize()
    out = y.float().cpu().numpy()
    if hidden:
        return out, enc.hidden().cpu().numpy()
    return out


GRIDS = [(1, 6, 10), (1, 2, 2), (1, 14, 18), (2, 4, 4)]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_deterministic_isolated_and_batch_invariant(dtype):
    cfg = small(dtype)
    patches = W.packed_patches(cfg, GRIDS)
    cu, grid = W.metadata(GRIDS)
    enc, gw, layers = make_encoder(cfg, 1024)
    try:
        y0 = run(enc, cfg, patches, cu, grid)
        y1 = run(enc, cfg, patches, cu, grid)
        assert np.array_equal(y0, y1), "two calls on the same input must be bit-identical"
        # perturb item 2 only (tokens 64..315): every other item's rows must not change at all
        p2 = patches.copy()
        p2[64:316] = W.round_to_dtype(p2[64:316] * 0.5 + 0.25, cfg.dtype)
        y2 = run(enc, cfg, p2, cu, grid)
        rows = np.cumsum([0] + [W.num_merged_tokens([g]) for g in GRIDS])
        for i in (0, 1, 3):
            assert np.array_equal(y0[rows[i]:rows[i + 1]], y2[rows[i]:rows[i + 1]]), "item %d changed" % i
        assert np.abs(y0[rows[2]:rows[3]] - y2[rows[2]:rows[3]]).max() > 1e-3
        # every item alone (same handle, smaller call) equals its rows in the batch
        tok = 0
        for i, g in enumerate(GRIDS):
            n = W.num_tokens([g])
            cu1, g1 = W.metadata([g])
            yi = run(enc, cfg, patches[tok:tok + n], cu1, g1)
            mabs, cos, rel = error_metrics(yi, y0[rows[i]:rows[i + 1]])
            log("  item %d alone vs in batch: max_abs %.3e (bit-identical: %s)" % (i, mabs, mabs == 0.0))
            assert mabs <= (1e-5 if dtype == "f32" else 2e-2 * np.abs(yi).max())
            tok += n
    finally:
        enc.close()


def test_bad_metadata_is_rejected_and_handle_survives():
    from paper_2601_11590_amd import binding as B
    cfg = small("bf16")
    patches = W.packed_patches(cfg, GRIDS)
    cu, grid = W.metadata(GRIDS)
    enc, gw, layers = make_encoder(cfg, 512, segs=4, items=4)
    try:
        good = run(enc, cfg, patches, cu, grid)
        bad_cases = [
            (np.array([0, 60, 60, 316, 348], np.int32), grid, "increasing"),         # empty segment
            (np.array([0, 60, 64, 316, 340], np.int32), grid, "cu_seqlens"),          # wrong total
            (np.array([1, 60, 64, 316, 348], np.int32), grid, "cu_seqlens"),          # does not start at 0
            (cu, np.array([[1, 6, 10], [1, 2, 2], [1, 14, 18], [2, 4, 5]], np.int32), "divisible"),
            (cu, np.array([[1, 6, 10], [1, 2, 2], [1, 14, 18], [2, 4, 4], [1, 2, 2]], np.int32), "num_items"),
            (np.array([0, 348, 700], np.int32), np.array([[1, 6, 10], [1, 2, 2], [1, 14, 18], [2, 4, 4], ], np.int32), "cu_seqlens"),
        ]
        for cu_b, grid_b, needle in bad_cases:
            with pytest.raises(B.EpdError) as ei:
                run(enc, cfg, patches, cu_b, grid_b)
            assert ei.value.status == B.EPD_ERR_SHAPE, str(ei.value)
            assert needle in str(ei.value), str(ei.value)
        # more tokens than the handle was sized for
        big = [(1, 20, 30)]
        with pytest.raises(B.EpdError) as ei:
            run(enc, cfg, W.packed_patches(cfg, big), *W.metadata(big))
        assert ei.value.status == B.EPD_ERR_SHAPE and "max_tokens" in str(ei.value)
        again = run(enc, cfg, patches, cu, grid)
        assert np.array_equal(good, again)
    finally:
        enc.close()


def test_smallest_inputs_and_single_token_segments():
    # one 2x2 item (4 tokens -> 1 visual token) and per-token segments (attention = identity on V)
    for dtype in ("f32", "bf16"):
        cfg = small(dtype)
        grids = [(1, 2, 2)]
        gw, layers = W.all_weights(cfg)
        patches = W.packed_patches(cfg, grids)
        for cu in (np.array([0, 4], np.int32), np.array([0, 1, 2, 3, 4], np.int32)):
            grid = np.array(grids, np.int32)
            ref = O.encode(cfg, gw, layers, patches, cu, grid)
            enc, _, _ = make_encoder(cfg, 4, segs=4, items=1)
            try:
                got = run(enc, cfg, patches, cu, grid)
            finally:
                enc.close()
            assert got.shape == (1, cfg.out_dim)
            check(cfg, got, ref, "segments=%d" % (len(cu) - 1))


def test_permutation_equivariance_without_rotary_on_gpu():
    cfg = small("bf16", rope="none", rope_pairs=(0, 0, 0))
    grids = [(1, 8, 8), (1, 4, 4)]
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids)
    enc, gw, layers = make_encoder(cfg, 128)
    try:
        _, h0 = run(enc, cfg, patches, cu, grid, hidden=True)
        perm = np.arange(80)
        perm[:64] = np.random.default_rng(1).permutation(64)
        _, h1 = run(enc, cfg, patches[perm], cu, grid, hidden=True)
    finally:
        enc.close()
    mabs, cos, rel = error_metrics(h1, h0[perm])
    log("  permuted hidden vs permutation of hidden: max_abs %.3e min_cos %.6f" % (mabs, cos))
    assert cos >= 0.9999 and rel <= 5e-3


def shaped_case(cfg, grids, what):
    log("case %s: %s" % (cfg.name, what))
    gw, layers = W.all_weights(cfg)
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids)
    ref = O.encode(cfg, gw, layers, patches, cu, grid)
    from parity_util import run_gpu
    got = run_gpu(cfg, gw, layers, patches, cu, grid)
    return check(cfg, got, ref, what)


def test_c3_width_varlen_one_layer():
    # first six images of the canonical varlen batch: 384 ... 5904 tokens per segment
    shaped_case(W.C3.replace(num_layers=1), W.grids_for(W.C3)[:6], "6 varlen images, L=1")


def test_c4_shape_head_dim_72_one_layer():
    # hidden 1152 = 16 x 72, MLP 4304 (K tail of 16), one 1344 x 1344 image = 7056 tokens
    shaped_case(W.C4.replace(num_layers=1), [(1, 84, 84)], "d=72, 7056-token single sequence, L=1")


def test_c5_shape_video_3d_rotary_one_layer():
    # hidden 3200 = 25 x 128, MLP 12800, patch 14 x temporal 2 (K = 1176, tail of 24), 3-D rotary
    shaped_case(W.C5.replace(num_layers=1), [(4, 16, 16), (2, 16, 32)], "video clips, L=1")


def test_c2_full_depth_batch_sampled_against_oracle():
    """The benchmark configuration as bench.py launches it (8 images, 24 layers); the oracle
    recomputes the first and the last image alone, which block-diagonal attention makes equal
    to their rows in the batch."""
    from paper_2601_11590_amd import binding as B
    import torch
    cfg = W.C2
    grids = W.grids_for(cfg)
    gw, layers = W.all_weights(cfg)
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids)
    enc = B.EpdEncoder(cfg, gw, layers, max_tokens=patches.shape[0], max_segments=8, max_items=8)
    try:
        got = enc.encode(B.to_device_patches(patches, cfg.dtype), cu, grid)
        torch.cuda.synchronize()
        got = got.float().cpu().numpy()
    finally:
        enc.close()
    assert got.shape == (1568, 4096) and np.isfinite(got).all()
    for item in (0, 7):
        cu1, g1 = W.metadata([grids[item]])
        ref = O.encode(cfg, gw, layers, patches[784 * item:784 * (item + 1)], cu1, g1)
        check(cfg, got[196 * item:196 * (item + 1)], ref, "image %d of 8, 24 layers" % item)


def test_empty_or_zero_sized_calls_are_rejected():
    from paper_2601_11590_amd import binding as B
    cfg = small("bf16")
    enc, gw, layers = make_encoder(cfg, 64, segs=2, items=2)
    try:
        import torch
        p = torch.zeros((4, cfg.patch_dim), dtype=torch.bfloat16, device="cuda:0")
        out = torch.zeros((1, cfg.out_dim), dtype=torch.bfloat16, device="cuda:0")
        import ctypes as C
        cu = (C.c_int32 * 2)(0, 4)
        grid = (C.c_int32 * 3)(1, 2, 2)
        st = B.lib.epd_encode(enc.handle, p.data_ptr(), C.cast(cu, C.POINTER(C.c_int32)), 0,
                              C.cast(grid, C.POINTER(C.c_int32)), 1, out.data_ptr(), None)
        assert st == B.EPD_ERR_SHAPE
        st = B.lib.epd_encode(enc.handle, p.data_ptr(), C.cast(cu, C.POINTER(C.c_int32)), 1,
                              C.cast(grid, C.POINTER(C.c_int32)), 0, out.data_ptr(), None)
        assert st == B.EPD_ERR_SHAPE
        st = B.lib.epd_encode(enc.handle, None, C.cast(cu, C.POINTER(C.c_int32)), 1,
                              C.cast(grid, C.POINTER(C.c_int32)), 1, out.data_ptr(), None)
        assert st == B.EPD_ERR_INVALID_ARG
        with pytest.raises(B.EpdError):
            B.epd_encode_debug_hidden(enc.handle, out.data_ptr(), 0)   # no completed call yet
    finally:
        enc.close()


def test_tuning_hook_rejects_what_has_no_kernel_and_keeps_the_result_within_tolerance():
    from paper_2601_11590_amd import binding as B
    cfg = small("bf16", num_heads=2, head_dim=128, rope="3d", rope_pairs=(16, 24, 24))
    enc, gw, layers = make_encoder(cfg, 512)
    try:
        for tile, groups, status in ((3, 0, B.EPD_ERR_INVALID_ARG), (-2, 0, B.EPD_ERR_INVALID_ARG), (0, 3, B.EPD_ERR_INVALID_ARG),
                                     (1, 0, B.EPD_ERR_INVALID_ARG), (-1, -1, B.EPD_ERR_INVALID_ARG)):
            with pytest.raises(B.EpdError) as ei:
                enc.set_tuning(tile, groups)
            assert ei.value.status == status, str(ei.value)
        patches = W.packed_patches(cfg, GRIDS)
        cu, grid = W.metadata(GRIDS)
        ref = O.encode(cfg, gw, layers, patches, cu, grid)
        auto = run(enc, cfg, patches, cu, grid)
        enc.set_tuning(2, 1)
        forced = run(enc, cfg, patches, cu, grid)
        enc.set_tuning(-1, 0)
        again = run(enc, cfg, patches, cu, grid)
        check(cfg, auto, ref, "automatic")
        check(cfg, forced, ref, "tile 256x128 forced")
        assert np.array_equal(auto, again), "switching the hook off must restore the first result bit for bit"
    finally:
        enc.close()


def test_compute_unit_hint_changes_launch_plans_only():
    # the hint for CU-masked streams (co-location): other tile plans, the same result within the
    # tolerances; values outside 0 .. 4096 are refused and change nothing
    from paper_2601_11590_amd import binding as B
    cfg = small("bf16", hidden=512, num_heads=8, mlp_dim=1088)
    enc, gw, layers = make_encoder(cfg, 512)
    try:
        patches = W.packed_patches(cfg, GRIDS)
        cu, grid = W.metadata(GRIDS)
        ref = O.encode(cfg, gw, layers, patches, cu, grid)
        whole = run(enc, cfg, patches, cu, grid)
        for n in (1, 7, 224):
            enc.set_compute_units(n)
            check(cfg, run(enc, cfg, patches, cu, grid), ref, "%d compute units" % n)
        for bad in (-1, 4097):
            with pytest.raises(B.EpdError) as ei:
                enc.set_compute_units(bad)
            assert ei.value.status == B.EPD_ERR_INVALID_ARG
        enc.set_compute_units(0)
        assert np.array_equal(whole, run(enc, cfg, patches, cu, grid)), "0 restores the plans for the whole device"
    finally:
        enc.close()


def test_c3_full_varlen_batch_one_layer():
    # all 32 images, 73 896 tokens (the maximum batch of the benchmark configurations), one layer
    shaped_case(W.C3.replace(num_layers=1), W.grids_for(W.C3), "32 varlen images, 73896 tokens, L=1")


def test_c4_full_sequence_one_layer():
    # one 2688 x 2688 image: a single 28 224-token segment, head dim 72
    shaped_case(W.C4.replace(num_layers=1), W.grids_for(W.C4), "28224-token single sequence, L=1")


def test_c5_full_video_batch_one_layer_last_clip_against_oracle():
    """All four 8 x 32 x 32 clips (32 768 tokens, hidden 3200, 25 x 128 heads, 3-D rotary) in one
    call, one layer; the oracle recomputes the last clip alone (8192-token segment), which
    block-diagonal attention makes equal to its rows in the batch."""
    from paper_2601_11590_amd import binding as B
    import torch
    cfg = W.C5.replace(num_layers=1)
    grids = W.grids_for(W.C5)
    log("case %s: 4 clips, 32768 tokens, L=1; oracle on the last clip" % cfg.name)
    gw, layers = W.all_weights(cfg)
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids)
    enc = B.EpdEncoder(cfg, gw, layers, max_tokens=patches.shape[0], max_segments=len(grids), max_items=len(grids))
    try:
        got = enc.encode(B.to_device_patches(patches, cfg.dtype), cu, grid)
        torch.cuda.synchronize()
        got = got.float().cpu().numpy()
    finally:
        enc.close()
    n, nm = W.num_tokens(grids[:1]), W.num_merged_tokens(grids[:1], cfg.merge)
    assert got.shape == (4 * nm, cfg.out_dim) and np.isfinite(got).all()
    cu1, g1 = W.metadata(grids[3:])
    ref = O.encode(cfg, gw, layers, patches[3 * n:], cu1, g1)
    check(cfg, got[3 * nm:], ref, "clip 4 of 4, 8192 tokens")


def test_c5_full_video_batch_one_layer_per_frame_segments_last_clip_against_oracle():
    """The video batch with one attention segment per frame (windowed attention: 32 segments of
    1024 tokens instead of 4 of 8192; rotary coordinates still run over the whole clip), one layer;
    the oracle recomputes the last clip with the same per-frame segments."""
    from paper_2601_11590_amd import binding as B
    import torch
    cfg = W.C5.replace(num_layers=1)
    grids = W.grids_for(W.C5)
    log("case %s: 4 clips, per-frame segments, L=1; oracle on the last clip" % cfg.name)
    gw, layers = W.all_weights(cfg)
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids, "frame")
    assert len(cu) - 1 == 32 and int(cu[1]) == 1024
    enc = B.EpdEncoder(cfg, gw, layers, max_tokens=patches.shape[0], max_segments=len(cu) - 1, max_items=len(grids))
    try:
        got = enc.encode(B.to_device_patches(patches, cfg.dtype), cu, grid)
        torch.cuda.synchronize()
        got = got.float().cpu().numpy()
    finally:
        enc.close()
    n, nm = W.num_tokens(grids[:1]), W.num_merged_tokens(grids[:1], cfg.merge)
    cu1, g1 = W.metadata(grids[3:], "frame")
    ref = O.encode(cfg, gw, layers, patches[3 * n:], cu1, g1)
    check(cfg, got[3 * nm:], ref, "clip 4 of 4, 8 frame segments of 1024 tokens")


def oracle_rows_one_layer(cfg, gw, lw, patches, cu, grid, merged_rows):
    """Rows `merged_rows` of the one-layer encoder's output, computed one window at a time from
    the oracle's own functions: keys and values of the whole batch (three matrix products), then
    for every sampled visual token the softmax rows of its merge x merge source tokens only."""
    H, d, D = cfg.num_heads, cfg.head_dim, cfg.hidden
    x = O.linear(patches, gw["patch_w"], gw.get("patch_b"))
    a = O.norm(cfg, x, lw["norm1_g"], lw.get("norm1_b"))
    theta = O.rotary_angles(O.token_coords(grid), cfg.rope_pairs, cfg.rope_base) if cfg.rope != "none" else None
    wq, wk, wv = lw["qkv_w"][:D], lw["qkv_w"][D:2 * D], lw["qkv_w"][2 * D:]
    bq, bk, bv = (lw["qkv_b"][i * D:(i + 1) * D] for i in range(3)) if "qkv_b" in lw else (None, None, None)
    T = x.shape[0]
    k = O.linear(a, wk, bk).reshape(T, H, d)
    v = O.linear(a, wv, bv).reshape(T, H, d)
    if theta is not None:
        k = O.apply_rotary(k, theta)
    idx = O.merge_gather_index(grid, cfg.merge)[merged_rows]                 # [rows, merge^2] source tokens
    tok = np.unique(idx.ravel())
    q = O.linear(a[tok], wq, bq).reshape(len(tok), H, d)
    if theta is not None:
        q = O.apply_rotary(q, theta[tok])
    seg = np.searchsorted(np.asarray(cu), tok, side="right") - 1
    o = np.zeros((len(tok), H, d))
    for i, t in enumerate(tok):
        s0, s1 = int(cu[seg[i]]), int(cu[seg[i] + 1])
        for h in range(H):
            p = O.softmax_rows((q[i:i + 1, h] @ k[s0:s1, h].T) / np.sqrt(float(d)))
            o[i, h] = p @ v[s0:s1, h]
    xs = x[tok] + O.linear(o.reshape(len(tok), D), lw["proj_w"], lw.get("proj_b"))
    b = O.norm(cfg, xs, lw["norm2_g"], lw.get("norm2_b"))
    xs = xs + O.linear(O.activation(cfg, O.linear(b, lw["fc1_w"], lw.get("fc1_b"))), lw["fc2_w"], lw.get("fc2_b"))
    z = O.norm(cfg, xs, gw["final_norm_g"], gw.get("final_norm_b"))
    pos = {int(t): i for i, t in enumerate(tok)}
    g = np.stack([np.concatenate([z[pos[int(t)]] for t in row]) for row in idx])
    return O.linear(g, gw["merge_w"], gw.get("merge_b"))


def test_oracle_rows_one_layer_helper_equals_the_oracle():
    # the sampled-row evaluation used below for sequences too long for the full oracle, checked
    # against the full oracle on a batch it can do (CPU arithmetic only)
    cfg = small("bf16", num_layers=1, norm="layernorm", num_heads=2, head_dim=72, hidden=144, rope_pairs=(0, 18, 18))
    gw, layers = W.all_weights(cfg)
    patches = W.packed_patches(cfg, GRIDS)
    cu, grid = W.metadata(GRIDS)
    ref = O.encode(cfg, gw, layers, patches, cu, grid)
    rows = np.array([0, 3, 14, 15, 16, 40, ref.shape[0] - 1])
    assert np.abs(oracle_rows_one_layer(cfg, gw, layers[0], patches, cu, grid, rows) - ref[rows]).max() < 1e-10


def test_table_4_2_batch_token_counts_and_parity():
    """The six resolutions of the paper's Table 4_2 (section 4.2) as one packed batch at patch 14
    (85 500 patch tokens, segments of 400 ... 64 824 tokens), one layer.  The library's output has
    one row per visual token: per image that is the count the table prints (100, 400, 1196, 2691,
    16 206; 782 by the rule for the inconsistent 640 x 960 row).  The five smaller images are
    compared with the oracle in full, the 64 824-token image on sampled rows."""
    from paper_2601_11590_amd import binding as B
    import torch
    cfg = W.T42.replace(num_layers=1)
    grids = W.grids_for(W.T42)
    log("case %s: %s, L=1" % (cfg.name, grids))
    gw, layers = W.all_weights(cfg)
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids)
    enc = B.EpdEncoder(cfg, gw, layers, max_tokens=patches.shape[0], max_segments=len(grids), max_items=len(grids))
    try:
        got = enc.encode(B.to_device_patches(patches, cfg.dtype), cu, grid)
        torch.cuda.synchronize()
        got = got.float().cpu().numpy()
    finally:
        enc.close()
    counts = [W.num_merged_tokens([g], cfg.merge) for g in grids]
    assert counts == [100, 400, 782, 1196, 2691, 16206]
    assert got.shape == (sum(counts), 3584) and np.isfinite(got).all()
    n5 = W.num_tokens(grids[:5])
    cu5, g5 = W.metadata(grids[:5])
    ref5 = O.encode(cfg, gw, layers, patches[:n5], cu5, g5)
    check(cfg, got[:sum(counts[:5])], ref5, "images 1-5 (280^2 ... 1080 x 1920)")
    first = sum(counts[:5])
    rows = first + np.unique(np.round(np.linspace(0, counts[5] - 1, 24)).astype(np.int64))
    ref6 = oracle_rows_one_layer(cfg, gw, layers[0], patches, cu, grid, rows)
    check(cfg, got[rows], ref6, "image 6 (4096 x 3112, 64824 tokens), %d sampled rows" % len(rows))


def test_c3_full_depth_varlen_batch_smallest_images_against_oracle():
    """The largest batch of the benchmark configurations at its full depth (32 images of mixed
    sizes, 73 896 tokens, 24 layers) in one call; the oracle recomputes the three smallest
    images alone, which block-diagonal attention makes equal to their rows in the batch."""
    from paper_2601_11590_amd import binding as B
    import torch
    cfg = W.C3
    grids = W.grids_for(cfg)
    log("case %s: 32 images, %d tokens, L=%d; oracle on the three smallest" % (cfg.name, W.num_tokens(grids), cfg.num_layers))
    gw, layers = W.all_weights(cfg)
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids)
    enc = B.EpdEncoder(cfg, gw, layers, max_tokens=patches.shape[0], max_segments=len(grids), max_items=len(grids))
    try:
        got = enc.encode(B.to_device_patches(patches, cfg.dtype), cu, grid)
        torch.cuda.synchronize()
        got = got.float().cpu().numpy()
    finally:
        enc.close()
    assert got.shape == (W.num_merged_tokens(grids), cfg.out_dim) and np.isfinite(got).all()
    toks = [t * h * w for t, h, w in grids]
    tok_off = np.concatenate([[0], np.cumsum(toks)])
    for item in np.argsort(toks, kind="stable")[:3]:
        cu1, g1 = W.metadata([grids[item]])
        ref = O.encode(cfg, gw, layers, patches[tok_off[item]:tok_off[item + 1]], cu1, g1)
        m0 = tok_off[item] // 4
        check(cfg, got[m0:m0 + toks[item] // 4], ref, "image %d (%d tokens) of 32, 24 layers" % (item, toks[item]))


def test_batches_in_flight_on_separate_streams_equal_the_single_stream_result():
    """Serving mode of bench.py (--in-flight): several encoders, each with its own workspace, take
    batches in turn on streams of their own, so kernels of different batches overlap on the GPU.
    Every call must return exactly what the same call returns alone."""
    from paper_2601_11590_amd import binding as B
    import torch
    cfg = W.C2.replace(num_layers=3)
    grids = W.grids_for(W.C2)
    gw, layers = W.all_weights(cfg)
    patches = B.to_device_patches(W.packed_patches(cfg, grids), cfg.dtype)
    other = B.to_device_patches(W.packed_patches(cfg, grids, seed=123), cfg.dtype)
    cu, grid = W.metadata(grids)
    encs = [B.EpdEncoder(cfg, gw, layers, max_tokens=patches.shape[0], max_segments=8, max_items=8) for _ in range(3)]
    try:
        alone = [encs[0].encode(p, cu, grid).clone() for p in (patches, other)]
        torch.cuda.synchronize()
        streams = [torch.cuda.Stream() for _ in encs]
        outs = []
        for rep in range(4):
            for i, (e, st) in enumerate(zip(encs, streams)):
                with torch.cuda.stream(st):
                    outs.append(((rep + i) % 2, e.encode(other if (rep + i) % 2 else patches, cu, grid).clone()))
        torch.cuda.synchronize()
        for which, o in outs:
            assert torch.equal(o, alone[which])
    finally:
        for e in encs:
            e.close()
