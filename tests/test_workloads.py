"""Host-side checks of the seeded input generators (no arithmetic of the method)."""

import numpy as np
import torch

from paper_2601_11590_amd import workloads as W


def test_bf16_rounding_matches_library_rne():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(100000) * 10.0 ** rng.integers(-6, 6, 100000)).astype(np.float32)
    a[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]        # exact ties: to even
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = W.round_to_dtype(a, "bf16")
    assert np.array_equal(got, want)
    assert np.array_equal(W.bf16_bits_to_f32(W.bf16_bits(a)), want)
    assert W.round_to_dtype(a, "f32") is not None and np.array_equal(W.round_to_dtype(a, "f32"), a)


def test_patchify_element_order():
    c, tp, p, t, h, w = 2, 2, 3, 2, 2, 2
    px = np.arange(c * t * tp * h * p * w * p, dtype=np.float32).reshape(c, t * tp, h * p, w * p)
    rows = W.patchify(px, p, tp)
    assert rows.shape == (t * h * w, c * tp * p * p)
    # token (ti=1, r=0, c=1), element (channel 1, temporal 1, row 2, col 0)
    tok = (1 * h + 0) * w + 1
    el = ((1 * tp + 1) * p + 2) * p + 0
    assert rows[tok, el] == px[1, 1 * tp + 1, 0 * p + 2, 1 * p + 0]


def test_config_table_shapes():
    want = {"C1": (256, 1, 64), "C2": (6272, 8, 1568), "C3": (73896, 32, 18474),
            "C4": (28224, 1, 7056), "C5": (32768, 4, 8192), "T42": (85500, 6, 21375)}
    for key, cfg in W.CONFIGS.items():
        grids = W.grids_for(cfg)
        assert cfg.hidden == cfg.num_heads * cfg.head_dim
        assert sum(cfg.rope_pairs) == cfg.head_dim // 2
        cu, g = W.metadata(grids)
        assert (W.num_tokens(grids), len(grids), W.num_merged_tokens(grids)) == want[key]
        assert cu[0] == 0 and cu[-1] == want[key][0] and g.shape == (len(grids), 3)
    assert W.C1.patch_dim == 588 and W.C2.patch_dim == 768 and W.C5.patch_dim == 1176


def test_table_4_2_workload_reproduces_the_visual_token_counts_the_paper_prints():
    """The T42 batch is the six resolutions of the paper's Table 4_2 at patch 14 with a 2x2 merge;
    its per-image visual-token counts must be the table's (five consistent rows; the 640 x 960 row
    is inconsistent in the paper itself and follows the rule here)."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_table4_2_token_counts.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert [(int(r[0]), int(r[1])) for r in rows] == list(W.T42_SIZES_PX)
    grids = W.grids_for(W.T42)
    for r, g in zip(rows, grids):
        n = W.num_merged_tokens([g], W.T42.merge)
        if int(r[4]):
            assert n == int(r[2]), (r, g)
        else:
            assert n != int(r[2]) and n == 782
        assert int(r[3]) == W.T42.out_dim == 3584
    assert W.T42.patch == 14 and W.T42.patch_dim == 1176 and W.T42.head_dim == 72


def test_c3_canonical_sizes_follow_the_stated_draw():
    lens = [t * h * w for t, h, w in W.grids_for(W.C3)]
    assert min(lens) == 280 and max(lens) == 5904
    assert all(224 <= a <= 1344 and a % 32 == 0 for hw in W.C3_SIZES_PX for a in hw)
    draw = np.random.default_rng(1).integers(7, 43, size=(32, 2)) * 32
    assert [tuple(r) for r in draw.tolist()] == list(W.C3_SIZES_PX)


def test_weights_are_seeded_rounded_and_shaped():
    cfg = W.C2.replace(num_layers=1, hidden=64, num_heads=1, mlp_dim=128, out_dim=32)
    a, b = W.layer_weights(cfg, 0), W.layer_weights(cfg, 0)
    assert all(np.array_equal(a[k], b[k]) for k in a)
    assert "norm1_b" not in a and a["qkv_w"].shape == (192, 64)
    assert np.array_equal(W.round_to_dtype(a["fc1_w"], "bf16"), a["fc1_w"])
    assert abs(a["fc1_w"].std() - 0.02) < 2e-3 and abs(a["norm1_g"].mean() - 1.0) < 2e-2
    c = W.layer_weights(cfg, 1)
    assert not np.array_equal(a["qkv_w"], c["qkv_w"])
    g = W.global_weights(W.C1)
    assert g["patch_w"].shape == (256, 588) and g["merge_w"].shape == (512, 1024) and "final_norm_b" in g
    s = W.layer_weights(cfg, 0, q_gain=16.0)
    assert np.allclose(s["qkv_w"][:64], W.round_to_dtype(a_raw_q(cfg) * 16, "bf16"))
    assert np.array_equal(s["qkv_w"][64:], a["qkv_w"][64:])


def a_raw_q(cfg):
    rng = np.random.default_rng([cfg.seed, 2, 1, 2])
    return (rng.standard_normal((3 * cfg.hidden, cfg.hidden), dtype=np.float32) * np.float32(0.02))[: cfg.hidden]


def test_pixels_uniform_unit_interval():
    px = W.item_pixels(W.C1, 0, (1, 16, 16))
    assert px.shape == (3, 1, 224, 224) and px.min() >= 0.0 and px.max() < 1.0
    assert abs(px.mean() - 0.5) < 0.01
    p = W.packed_patches(W.C1, [(1, 16, 16)])
    assert p.shape == (256, 588)


def test_raw_uint8_pixels_are_seeded_sized_and_use_the_whole_byte_range():
    a = W.item_pixels_u8(W.C5, 2, (2, 4, 6))
    assert a.dtype == np.uint8 and a.shape == (3, 4, 56, 84)            # frames = t * temporal_patch, grid size in pixels
    assert np.array_equal(a, W.item_pixels_u8(W.C5, 2, (2, 4, 6)))
    assert not np.array_equal(a, W.item_pixels_u8(W.C5, 3, (2, 4, 6)))
    b = W.item_pixels_u8(W.C2, 0, (1, 28, 28), src_hw=(300, 500))
    assert b.shape == (3, 1, 300, 500) and b.min() == 0 and b.max() == 255
    # neighbouring pixels are correlated (a smooth pattern under the noise)
    d = np.abs(np.diff(b[0, 0].astype(np.int32), axis=1)).mean()
    assert d < 0.6 * np.abs(b[0, 0].astype(np.int32) - np.roll(b[0, 0].astype(np.int32), 97, axis=1)).mean()
