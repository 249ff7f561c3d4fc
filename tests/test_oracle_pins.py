"""Pins for the CPU oracle (oracle/vit_encode.py) against things other than itself:
scalar brute force, closed forms, invariants, library special cases and the token counts
the paper prints in Table 4_2.  CPU only."""

import math
import os
import types

import numpy as np
import pytest
import torch

from oracle import brute_force, vit_encode as O
from paper_2601_11590_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(**kw):
    base = dict(name="tiny", dtype="f32", num_layers=2, hidden=16, num_heads=2, head_dim=8,
                mlp_dim=24, patch=2, temporal_patch=1, norm="layernorm", rope="3d",
                rope_pairs=(1, 1, 2), out_dim=12, in_channels=1, seed=7)
    base.update(kw)
    return W.EncoderConfig(**base)


def tiny_case(cfg, grids, std=0.3, segments="item", seed=None):
    gw, layers = W.all_weights(cfg, std=std)
    patches = W.packed_patches(cfg, grids, seed)
    cu, grid = W.metadata(grids, segments)
    return gw, layers, patches, cu, grid


# ------------------------------------------------------------------ brute force

@pytest.mark.parametrize("norm,rope,pairs,act,segments", [
    ("layernorm", "3d", (1, 1, 2), "gelu_erf", "item"),
    ("rmsnorm", "2d", (0, 2, 2), "gelu_tanh", "item"),
    ("rmsnorm", "3d", (2, 1, 1), "gelu_erf", "frame"),
    ("layernorm", "none", (0, 0, 0), "gelu_erf", "item"),
])
def test_whole_encoder_matches_scalar_brute_force(norm, rope, pairs, act, segments):
    cfg = tiny_cfg(norm=norm, rope=rope, rope_pairs=pairs, act=act)
    grids = [(1, 2, 4), (2, 2, 2), (1, 4, 2)]
    gw, layers, patches, cu, grid = tiny_case(cfg, grids, segments=segments)
    y = O.encode(cfg, gw, layers, patches, cu, grid)
    yb = np.asarray(brute_force.encode(cfg, gw, layers, patches, cu, grid))
    assert y.shape == yb.shape == (W.num_merged_tokens(grids), cfg.out_dim)
    assert np.abs(yb).max() > 1e-2
    np.testing.assert_allclose(y, yb, rtol=0, atol=1e-10)


def test_attention_matches_brute_force_per_element():
    rng = np.random.default_rng(3)
    T, H, d = 23, 3, 6
    q, k, v = (rng.standard_normal((T, H, d)) * 2.0 for _ in range(3))
    cu = [0, 5, 6, 17, 23]
    o = O.attention_varlen(q, k, v, cu, slab=4)
    ob = np.asarray(brute_force.attention(q.tolist(), k.tolist(), v.tolist(), cu))
    np.testing.assert_allclose(o, ob, rtol=0, atol=1e-12)


# ------------------------------------------------------------------ attention invariants

def test_softmax_rows_sum_to_one_and_special_cases():
    rng = np.random.default_rng(4)
    T, H, d = 40, 2, 8
    q, k, v = (rng.standard_normal((T, H, d)) * 3.0 for _ in range(3))
    cu = [0, 1, 14, 40]
    o, probs = O.attention_varlen(q, k, v, cu, slab=7, return_probs=True)
    for p, n in zip(probs, (1, 13, 26)):
        assert p.shape == (H, n, n)
        assert np.abs(p.sum(axis=-1) - 1.0).max() < 1e-12
        assert p.min() >= 0.0
    # segment of length one: output is its own value row
    np.testing.assert_allclose(o[0], v[0], atol=1e-15)
    # zero queries: uniform weights -> mean of the segment's values
    o0 = O.attention_varlen(np.zeros_like(q), k, v, cu)
    np.testing.assert_allclose(o0[1:14], np.broadcast_to(v[1:14].mean(0), (13, H, d)), atol=1e-13)
    np.testing.assert_allclose(o0[14:], np.broadcast_to(v[14:].mean(0), (26, H, d)), atol=1e-13)
    # constant values: constant output
    vc = np.ones_like(v) * 1.75
    np.testing.assert_allclose(O.attention_varlen(q, k, vc, cu), vc, atol=1e-13)


def test_attention_overflow_safe_with_huge_logit():
    rng = np.random.default_rng(5)
    T, H, d = 12, 1, 4
    q, k, v = (rng.standard_normal((T, H, d)) for _ in range(3))
    q[:, 0, 0] = 400.0
    k[3, 0, 0] = 50.0        # logit ~ 400*50/2 = 1e4 on key 3: exp would overflow without max shift
    o = O.attention_varlen(q, k, v, [0, T])
    assert np.isfinite(o).all()
    np.testing.assert_allclose(o[:, 0], np.broadcast_to(v[3, 0], (T, d)), atol=1e-9)


def test_attention_matches_library_sdpa_per_segment():
    rng = np.random.default_rng(6)
    T, H, d = 50, 4, 16
    q, k, v = (rng.standard_normal((T, H, d)) for _ in range(3))
    cu = [0, 9, 30, 50]
    o = O.attention_varlen(q, k, v, cu)
    for a, b in zip(cu[:-1], cu[1:]):
        tq, tk, tv = (torch.from_numpy(x[a:b]).permute(1, 0, 2)[None] for x in (q, k, v))
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].permute(1, 0, 2)
        np.testing.assert_allclose(o[a:b], ref.numpy(), atol=1e-12)


# ------------------------------------------------------------------ structure of the encoder

def test_block_diagonal_isolation_bitwise():
    cfg = tiny_cfg()
    grids = [(1, 2, 2), (1, 4, 2), (2, 2, 2)]
    gw, layers, patches, cu, grid = tiny_case(cfg, grids)
    y0 = O.encode(cfg, gw, layers, patches, cu, grid)
    p2 = patches.copy()
    p2[4:12] += 0.5                     # item 1 only (tokens 4..11)
    y1 = O.encode(cfg, gw, layers, p2, cu, grid)
    # merged rows: item0 -> 1 row, item1 -> 2 rows, item2 -> 2 rows
    assert np.array_equal(y0[:1], y1[:1]) and np.array_equal(y0[3:], y1[3:])
    assert np.abs(y0[1:3] - y1[1:3]).max() > 1e-3


def test_batch_equals_each_item_alone():
    cfg = tiny_cfg(norm="rmsnorm", rope="2d", rope_pairs=(0, 2, 2))
    grids = [(1, 4, 4), (1, 2, 6), (1, 4, 4)]
    gw, layers, patches, cu, grid = tiny_case(cfg, grids)
    y = O.encode(cfg, gw, layers, patches, cu, grid)
    row, tok = 0, 0
    for g in grids:
        n, nm = W.num_tokens([g]), W.num_merged_tokens([g])
        cu1, g1 = W.metadata([g])
        y1 = O.encode(cfg, gw, layers, patches[tok:tok + n], cu1, g1)
        np.testing.assert_allclose(y[row:row + nm], y1, rtol=0, atol=1e-13)
        row, tok = row + nm, tok + n


def test_permutation_equivariance_without_rotary():
    cfg = tiny_cfg(rope="none", rope_pairs=(0, 0, 0))
    grids = [(1, 4, 4), (1, 2, 2)]
    gw, layers, patches, cu, grid = tiny_case(cfg, grids)
    _, h0 = O.encode(cfg, gw, layers, patches, cu, grid, return_hidden=True)
    perm = np.arange(20)
    perm[:16] = np.random.default_rng(0).permutation(16)      # shuffle inside segment 0 only
    _, h1 = O.encode(cfg, gw, layers, patches[perm], cu, grid, return_hidden=True)
    np.testing.assert_allclose(h1, h0[perm], rtol=0, atol=1e-12)
    # with rotary the same shuffle must change the result (the position signal is real)
    cfg_r = tiny_cfg(rope="2d", rope_pairs=(0, 2, 2))
    _, r0 = O.encode(cfg_r, gw, layers, patches, cu, grid, return_hidden=True)
    _, r1 = O.encode(cfg_r, gw, layers, patches[perm], cu, grid, return_hidden=True)
    assert np.abs(r1 - r0[perm]).max() > 1e-4


def test_segments_need_not_coincide_with_items():
    # per-frame segments of a clip: each frame's tokens must equal the frame run as its own item
    # when the temporal rotary axis is unused (so coordinates agree).
    cfg = tiny_cfg(rope="2d", rope_pairs=(0, 2, 2))
    gw, layers = W.all_weights(cfg, std=0.3)
    grids = [(3, 2, 4)]
    patches = W.packed_patches(cfg, grids)
    cu, grid = W.metadata(grids, "frame")
    assert cu.tolist() == [0, 8, 16, 24]
    y = O.encode(cfg, gw, layers, patches, cu, grid)
    for f in range(3):
        cu1, g1 = W.metadata([(1, 2, 4)])
        y1 = O.encode(cfg, gw, layers, patches[8 * f:8 * f + 8], cu1, g1)
        np.testing.assert_allclose(y[2 * f:2 * f + 2], y1, atol=1e-13)


# ------------------------------------------------------------------ rotary

def test_rotary_identity_norm_and_translation_invariance():
    rng = np.random.default_rng(8)
    pairs, base = (2, 3, 3), 100.0
    coords = np.array([[0, 0, 0], [1, 2, 3], [4, 0, 7], [2, 5, 1]])
    th = O.rotary_angles(coords, pairs, base)
    assert th.shape == (4, 8)
    x = rng.standard_normal((4, 2, 16))
    xr = O.apply_rotary(x, th)
    np.testing.assert_array_equal(xr[0], x[0])                      # origin: identity
    # every pair keeps its length
    n0 = x[..., :8] ** 2 + x[..., 8:] ** 2
    n1 = xr[..., :8] ** 2 + xr[..., 8:] ** 2
    np.testing.assert_allclose(n1, n0, atol=1e-13)
    # scores depend on coordinate differences only
    y = rng.standard_normal((4, 2, 16))
    s0 = np.einsum("thd,uhd->htu", O.apply_rotary(x, th), O.apply_rotary(y, th))
    th2 = O.rotary_angles(coords + np.array([[3, 11, 5]]), pairs, base)
    s1 = np.einsum("thd,uhd->htu", O.apply_rotary(x, th2), O.apply_rotary(y, th2))
    np.testing.assert_allclose(s1, s0, atol=1e-11)


def test_rotary_explicit_angles_and_axis_assignment():
    # pairs (1, 2, 1), base 100: angles must be [t*1, h*1, h*100^-0.5, w*1]
    th = O.rotary_angles(np.array([[2, 3, 5]]), (1, 2, 1), 100.0)
    np.testing.assert_allclose(th[0], [2.0, 3.0, 0.3, 5.0], atol=1e-15)
    # a single pair (x0, x1) = (1, 0) turned by +theta lands on (cos, sin)
    out = O.apply_rotary(np.array([[[1.0, 0.0]]]), np.array([[0.25]]))
    np.testing.assert_allclose(out[0, 0], [math.cos(0.25), math.sin(0.25)], atol=1e-15)
    # complex-number form of the same rotation: (x_p + i x_{p+half}) * exp(i theta)
    rng = np.random.default_rng(9)
    x = rng.standard_normal((5, 1, 12))
    th = rng.standard_normal((5, 6)) * 3
    z = (x[..., :6] + 1j * x[..., 6:]) * np.exp(1j * th)[:, None, :]
    np.testing.assert_allclose(O.apply_rotary(x, th), np.concatenate([z.real, z.imag], -1), atol=1e-13)


def test_whole_encoder_translation_invariance_hook():
    cfg = tiny_cfg()
    grids = [(2, 2, 2), (1, 2, 4)]
    gw, layers, patches, cu, grid = tiny_case(cfg, grids)
    y0 = O.encode(cfg, gw, layers, patches, cu, grid)
    y1 = O.encode(cfg, gw, layers, patches, cu, grid, coord_offset=(5, 9, 2))
    np.testing.assert_allclose(y1, y0, atol=1e-10)


# ------------------------------------------------------------------ norms, GELU

def test_norm_moments_scale_invariance_and_library():
    rng = np.random.default_rng(10)
    x = rng.standard_normal((7, 48)) * 3 + 1.5
    eps = 1e-6
    one = np.ones(48)
    y = O.layer_norm(x, one, None, eps)
    var = x.var(axis=-1)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-14)
    np.testing.assert_allclose(y.var(-1), var / (var + eps), rtol=1e-12)
    r = O.rms_norm(x, one, eps)
    ms = (x * x).mean(-1)
    np.testing.assert_allclose((r * r).mean(-1), ms / (ms + eps), rtol=1e-12)
    np.testing.assert_allclose(O.layer_norm(64.0 * x, one, None, 0.0), O.layer_norm(x, one, None, 0.0), atol=1e-12)
    np.testing.assert_allclose(O.rms_norm(64.0 * x, one, 0.0), O.rms_norm(x, one, 0.0), atol=1e-12)
    g, b = rng.standard_normal(48), rng.standard_normal(48)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b), eps)
    np.testing.assert_allclose(O.layer_norm(x, g, b, eps), ref.numpy(), atol=1e-12)
    # RMSNorm written from its definition with plain loops
    for i in range(2):
        want = [x[i, c] / math.sqrt(sum(v * v for v in x[i]) / 48 + eps) * g[c] for c in range(48)]
        np.testing.assert_allclose(O.rms_norm(x, g, eps)[i], want, rtol=1e-13)


def test_gelu_closed_form_values():
    assert O.gelu_erf(0.0) == 0.0
    x = np.linspace(-6, 6, 101)
    np.testing.assert_allclose(O.gelu_erf(x) - O.gelu_erf(-x), x, atol=1e-14)
    # GELU(1) = Phi(1), GELU(-1) = -(1 - Phi(1)), GELU(2) = 2 Phi(2): standard normal CDF table values
    assert abs(float(O.gelu_erf(1.0)) - 0.8413447460685429) < 1e-15
    assert abs(float(O.gelu_erf(-1.0)) + 0.15865525393145707) < 1e-15
    assert abs(float(O.gelu_erf(2.0)) - 2 * 0.9772498680518208) < 1e-14
    # the tanh form is a different function: it must not be what "gelu_erf" computes
    assert abs(float(O.gelu_tanh(1.0)) - 0.8411919906082768) < 1e-12
    assert abs(float(O.gelu_tanh(1.0)) - float(O.gelu_erf(1.0))) > 1e-4
    ref = torch.nn.functional.gelu(torch.from_numpy(x))
    np.testing.assert_allclose(O.gelu_erf(x), ref.numpy(), atol=1e-14)


# ------------------------------------------------------------------ closed form with no layers

def test_zero_layers_is_two_matmuls_and_a_gather():
    cfg = tiny_cfg(num_layers=0, final_norm=False)
    grids = [(1, 4, 6), (2, 2, 2)]
    gw, layers, patches, cu, grid = tiny_case(cfg, grids)
    y = O.encode(cfg, gw, [], patches, cu, grid)
    x = patches.astype(np.float64) @ gw["patch_w"].astype(np.float64).T + gw["patch_b"]
    # gather written independently: item 0 is a 4x6 grid, item 1 two 2x2 frames
    rows = []
    for i in range(2):
        for j in range(3):
            rows.append(np.concatenate([x[(2 * i) * 6 + 2 * j], x[(2 * i) * 6 + 2 * j + 1],
                                        x[(2 * i + 1) * 6 + 2 * j], x[(2 * i + 1) * 6 + 2 * j + 1]]))
    for f in range(2):
        b = 24 + 4 * f
        rows.append(np.concatenate([x[b], x[b + 1], x[b + 2], x[b + 3]]))
    want = np.stack(rows) @ gw["merge_w"].astype(np.float64).T + gw["merge_b"]
    np.testing.assert_allclose(y, want, atol=1e-13)
    # linear in the input (bias removed)
    y2 = O.encode(cfg, gw, [], 2.0 * patches, cu, grid)
    zero = O.encode(cfg, gw, [], 0.0 * patches, cu, grid)
    np.testing.assert_allclose(y2 - zero, 2.0 * (y - zero), atol=1e-12)


def test_merge_gather_order_with_token_index_rows():
    grid = [(1, 4, 4), (2, 2, 4)]
    idx = O.merge_gather_index(grid, 2)
    assert idx.shape == (4 + 4, 4)
    assert idx[0].tolist() == [0, 1, 4, 5]
    assert idx[1].tolist() == [2, 3, 6, 7]
    assert idx[2].tolist() == [8, 9, 12, 13]
    assert idx[4].tolist() == [16, 17, 20, 21]          # second item starts at token 16
    assert idx[6].tolist() == [24, 25, 28, 29]          # its second frame
    assert sorted(idx.ravel().tolist()) == list(range(32))
    z = np.arange(32, dtype=np.float64)[:, None] * np.ones((1, 3))
    g = O.merge_tokens(z, grid, 2)
    assert g.shape == (8, 12)
    assert g[1].tolist() == [2, 2, 2, 3, 3, 3, 6, 6, 6, 7, 7, 7]


def test_token_coords_raster_order():
    c = O.token_coords([(2, 2, 3), (1, 1, 2)])
    assert c.shape == (14, 3)
    assert c[0].tolist() == [0, 0, 0] and c[1].tolist() == [0, 0, 1]
    assert c[3].tolist() == [0, 1, 0] and c[6].tolist() == [1, 0, 0]
    assert c[11].tolist() == [1, 1, 2]
    assert c[12].tolist() == [0, 0, 0] and c[13].tolist() == [0, 0, 1]   # restart per item


# ------------------------------------------------------------------ the paper's own numbers

def test_merged_token_counts_match_paper_table_4_2():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "paper_table4_2_token_counts.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 6
    checked = 0
    for hp, wp, n, width, ok in (tuple(int(v) for v in r) for r in rows):
        gh, gw_ = 2 * int(round(hp / 28)), 2 * int(round(wp / 28))     # patch 14, 2x2 merge
        got = O.merged_token_count([(1, gh, gw_)], 2)
        if ok:
            assert got == n, (hp, wp, got, n)
            checked += 1
        else:
            assert got != n          # the 640x960 row is inconsistent in the paper itself
        assert width == 3584
    assert checked == 5


def test_output_shape_is_n_by_d_as_in_eq_1():
    cfg = tiny_cfg()
    grids = [(1, 2, 2), (1, 4, 2)]
    gw, layers, patches, cu, grid = tiny_case(cfg, grids)
    y = O.encode(cfg, gw, layers, patches, cu, grid)
    assert y.shape == (O.merged_token_count(grid), cfg.out_dim) == (3, 12)
    assert y.dtype == np.float64


# ------------------------------------------------------------------ planted mistakes are caught

@pytest.mark.parametrize("mistake", ["rot_sign", "no_scale", "pair_adjacent", "gather_colmajor", "unbiased_var"])
def test_pins_catch_planted_mistakes(mistake, monkeypatch):
    """Each plausible slip, planted in the oracle on the CPU, must break the brute-force pin."""
    cfg = tiny_cfg()
    grids = [(1, 2, 4), (2, 2, 2)]
    gw, layers, patches, cu, grid = tiny_case(cfg, grids)
    yb = np.asarray(brute_force.encode(cfg, gw, layers, patches, cu, grid))
    if mistake == "rot_sign":
        orig = O.apply_rotary
        monkeypatch.setattr(O, "apply_rotary", lambda x, th: orig(x, -th))
    elif mistake == "no_scale":
        orig = O.attention_varlen
        monkeypatch.setattr(O, "attention_varlen",
                            lambda q, k, v, cu_, **kw: orig(q * math.sqrt(q.shape[-1]), k, v, cu_, **kw))
    elif mistake == "pair_adjacent":
        def adj(x, th):
            c, s = np.cos(th)[:, None, :], np.sin(th)[:, None, :]
            a, b = x[..., 0::2], x[..., 1::2]
            out = np.empty_like(x)
            out[..., 0::2], out[..., 1::2] = a * c - b * s, a * s + b * c
            return out
        monkeypatch.setattr(O, "apply_rotary", adj)
    elif mistake == "gather_colmajor":
        orig = O.merge_gather_index
        monkeypatch.setattr(O, "merge_gather_index", lambda g, m=2: orig(g, m)[:, [0, 2, 1, 3]])
    elif mistake == "unbiased_var":
        def ln(x, g, b, eps):
            mu = x.mean(-1, keepdims=True)
            var = x.var(-1, keepdims=True, ddof=1)
            y = (x - mu) / np.sqrt(var + eps) * g
            return y if b is None else y + b
        monkeypatch.setattr(O, "layer_norm", ln)
    y = O.encode(cfg, gw, layers, patches, cu, grid)
    assert np.abs(y - yb).max() > 1e-6
