"""Pins of the preprocessing oracle (raw pixels -> packed patch rows; the input I_m of the
paper's Eq. 1) to things other than itself: the library's bilinear routine, closed forms,
invariants, and a scalar loop written per output element."""

import numpy as np
import pytest
import torch

from oracle import preprocess as P


def rng(seed):
    return np.random.default_rng(seed)


@pytest.mark.parametrize("hs,ws,ho,wo", [(7, 9, 14, 12), (20, 31, 8, 12), (16, 16, 16, 16), (5, 40, 28, 4), (1, 3, 6, 6)])
def test_resize_matches_the_library_bilinear_routine(hs, ws, ho, wo):
    f = rng(hs * 100 + ws).random((hs, ws))
    ref = torch.nn.functional.interpolate(torch.from_numpy(f)[None, None], size=(ho, wo), mode="bilinear",
                                          align_corners=False, antialias=False)[0, 0].numpy()
    np.testing.assert_allclose(P.resize_bilinear(f, ho, wo), ref, rtol=0, atol=1e-13)


def test_resize_to_equal_size_is_the_identity():
    f = rng(3).integers(0, 256, size=(12, 20)).astype(np.float64)
    assert np.array_equal(P.resize_bilinear(f, 12, 20), f)


def test_resize_is_exact_on_affine_images_away_from_the_clamped_border():
    hs, ws, ho, wo = 24, 36, 40, 20
    y, x = np.mgrid[0:hs, 0:ws].astype(np.float64)
    f = 3.0 + 0.25 * y - 0.5 * x
    got = P.resize_bilinear(f, ho, wo)
    sy = (np.arange(ho) + 0.5) * hs / ho - 0.5
    sx = (np.arange(wo) + 0.5) * ws / wo - 0.5
    want = 3.0 + 0.25 * sy[:, None] - 0.5 * sx[None, :]
    inside = (sy[:, None] >= 0) & (sy[:, None] <= hs - 1) & (sx[None, :] >= 0) & (sx[None, :] <= ws - 1)
    assert inside.sum() > 0.8 * ho * wo
    np.testing.assert_allclose(got[inside], want[inside], rtol=0, atol=1e-12)
    # a transposed or mirrored tap would break the sign of one slope
    assert got[10, 3] > got[10, 15] and got[30, 5] > got[5, 5]


def test_resize_keeps_constants_and_stays_inside_the_pixel_range():
    assert np.all(P.resize_bilinear(np.full((9, 5), 17.0), 33, 21) == 17.0)
    f = rng(5).integers(0, 256, size=(13, 11)).astype(np.float64)
    g = P.resize_bilinear(f, 30, 7)
    assert g.min() >= f.min() and g.max() <= f.max()


def test_source_coords_weights_of_a_twofold_upscale():
    # 2x upscale: samples sit at -0.25 (clamped to 0), 0.25, 0.75, 1.25, ...
    i0, i1, w1 = P.source_coords(8, 4)
    assert list(i0) == [0, 0, 0, 1, 1, 2, 2, 3]
    assert list(i1) == [1, 1, 1, 2, 2, 3, 3, 3]
    np.testing.assert_allclose(w1, [0, 0.25, 0.75, 0.25, 0.75, 0.25, 0.75, 0.25], atol=1e-15)


def test_normalise_closed_form_values():
    x = np.zeros((3, 1, 1, 2))
    x[..., 1] = 255.0
    got = P.normalise(x, mean=[0.5, 0.25, 0.0], std=[0.5, 0.25, 2.0])
    np.testing.assert_allclose(got[:, 0, 0, 0], [-1.0, -1.0, 0.0], atol=1e-15)
    np.testing.assert_allclose(got[:, 0, 0, 1], [1.0, 3.0, 0.5], atol=1e-15)


def test_patch_rows_order_by_scalar_loops():
    c, t, tp, h, w, p = 2, 2, 2, 3, 2, 4
    px = rng(7).random((c, t * tp, h * p, w * p))
    got = P.patch_rows(px, p, tp)
    assert got.shape == (t * h * w, c * tp * p * p)
    for ti in range(t):
        for r in range(h):
            for col in range(w):
                tok = (ti * h + r) * w + col
                for ci in range(c):
                    for dt in range(tp):
                        for py in range(p):
                            for pxx in range(p):
                                k = ((ci * tp + dt) * p + py) * p + pxx
                                assert got[tok, k] == px[ci, ti * tp + dt, r * p + py, col * p + pxx]


def scalar_preprocess(items, grids, p, tp, mean, std):
    """The whole function again, one output element at a time, straight from the definitions."""
    rows = []
    for px, (t, h, w) in zip(items, grids):
        c, frames, hs, ws = px.shape
        ho, wo = h * p, w * p
        out = np.zeros((t * h * w, c * tp * p * p))
        for tok in range(t * h * w):
            ti, r, col = tok // (h * w), (tok // w) % h, tok % w
            for k in range(c * tp * p * p):
                ci, dt, py, pxx = k // (tp * p * p), (k // (p * p)) % tp, (k // p) % p, k % p
                y, x = r * p + py, col * p + pxx
                sy = max((y + 0.5) * hs / ho - 0.5, 0.0)
                sx = max((x + 0.5) * ws / wo - 0.5, 0.0)
                y0, x0 = min(int(np.floor(sy)), hs - 1), min(int(np.floor(sx)), ws - 1)
                y1, x1 = min(y0 + 1, hs - 1), min(x0 + 1, ws - 1)
                fy, fx = sy - y0, sx - x0
                f = px[ci, ti * tp + dt].astype(np.float64)
                v = (1 - fy) * ((1 - fx) * f[y0, x0] + fx * f[y0, x1]) + fy * ((1 - fx) * f[y1, x0] + fx * f[y1, x1])
                out[tok, k] = (v / 255.0 - mean[ci]) / std[ci]
        rows.append(out)
    return np.concatenate(rows, axis=0)


def test_whole_function_against_scalar_loops_with_and_without_resize():
    p, tp = 4, 2
    grids = [(1, 2, 3), (2, 1, 2), (1, 2, 2)]
    src = [(8, 12), (7, 5), (19, 23)]           # equal size, upscale, downscale
    r = rng(11)
    items = [r.integers(0, 256, size=(3, t * tp, hs, ws), dtype=np.uint8) for (t, h, w), (hs, ws) in zip(grids, src)]
    mean, std = [0.48, 0.46, 0.41], [0.27, 0.26, 0.28]
    got = P.preprocess(items, grids, p, tp, mean, std)
    want = scalar_preprocess(items, grids, p, tp, mean, std)
    assert got.shape == want.shape == (6 + 4 + 4, 3 * tp * p * p)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    # first item is not resized: its rows are the normalised bytes themselves
    first = (items[0][0, 0, 0, 0] / 255.0 - mean[0]) / std[0]
    assert abs(got[0, 0] - first) < 1e-15
