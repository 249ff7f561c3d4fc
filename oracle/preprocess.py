"""CPU oracle of the step in front of the encoder: raw pixels I_m -> packed patch rows
(paper section 3.1: the Encode stage takes the multimodal input I_m itself, images and video,
and Eq. 1 maps it to V_m; the rows produced here are what the patch embedding multiplies).

TEST INFRASTRUCTURE ONLY.  Imported by the tests (and nothing of the product); shares no code
with the HIP path and imports nothing from the package.

The paper does not say how I_m becomes encoder input.  Readings taken here:
  * pixels arrive as uint8, planar [C, frames, Hs, Ws] per item (frames = t * temporal_patch);
  * every frame is resized to the item's grid, (h * patch) x (w * patch), by bilinear
    interpolation with half-pixel centres, source coordinates clamped to the image, no
    antialiasing filter; frames are not resampled in time; equal sizes leave pixels untouched;
  * normalisation is per channel, (v / 255 - mean_c) / std_c;
  * a patch row lists (channel, frame in patch, row in patch, column in patch), tokens in
    raster order over (t, h, w), items packed in order.
Everything is float64; nothing is blocked or fused.

Pins (tests/test_oracle_preprocess.py): the resize against the library's bilinear routine,
identity at equal sizes, exactness on affine images, constants, the closed-form normalised
values of 0 and 255, and a scalar loop written per output element for the whole function.
"""

from __future__ import annotations

import numpy as np

F64 = np.float64


def source_coords(n_out: int, n_in: int):
    """Bilinear taps along one axis: (i0, i1, w1) with value = (1 - w1) * p[i0] + w1 * p[i1].

    Output sample j sits at (j + 0.5) * n_in / n_out - 0.5 in source pixel units (pixel
    centres at integers), clamped below at 0; the upper neighbour is clamped to the last pixel.
    """
    j = np.arange(n_out, dtype=F64)
    s = (j + 0.5) * (F64(n_in) / F64(n_out)) - 0.5
    s = np.maximum(s, 0.0)
    i0 = np.minimum(np.floor(s).astype(np.int64), n_in - 1)
    i1 = np.minimum(i0 + 1, n_in - 1)
    w1 = s - i0
    return i0, i1, w1


def resize_bilinear(frame: np.ndarray, h_out: int, w_out: int) -> np.ndarray:
    """One frame [Hs, Ws] -> [h_out, w_out], float64."""
    f = np.asarray(frame, dtype=F64)
    y0, y1, wy = source_coords(h_out, f.shape[0])
    x0, x1, wx = source_coords(w_out, f.shape[1])
    top = f[y0][:, x0] * (1.0 - wx) + f[y0][:, x1] * wx
    bot = f[y1][:, x0] * (1.0 - wx) + f[y1][:, x1] * wx
    return top * (1.0 - wy)[:, None] + bot * wy[:, None]


def normalise(x: np.ndarray, mean, std) -> np.ndarray:
    """(v / 255 - mean_c) / std_c for x [C, ...] holding pixel values on the 0..255 scale."""
    x = np.asarray(x, dtype=F64)
    shape = (-1,) + (1,) * (x.ndim - 1)
    return (x / 255.0 - np.asarray(mean, dtype=F64).reshape(shape)) / np.asarray(std, dtype=F64).reshape(shape)


def patch_rows(pixels: np.ndarray, patch: int, temporal_patch: int) -> np.ndarray:
    """[C, t*tp, h*p, w*p] -> [t*h*w, C*tp*p*p]: token (ti, r, c) raster order, element order
    (channel, frame in patch, row in patch, column in patch)."""
    c, tt, hh, ww = pixels.shape
    t, h, w = tt // temporal_patch, hh // patch, ww // patch
    x = pixels.reshape(c, t, temporal_patch, h, patch, w, patch)
    x = x.transpose(1, 3, 5, 0, 2, 4, 6)
    return np.ascontiguousarray(x.reshape(t * h * w, c * temporal_patch * patch * patch))


def preprocess(items, grid_thw, patch: int, temporal_patch: int, mean, std) -> np.ndarray:
    """items[i]: uint8 [C, t_i*tp, Hs_i, Ws_i]; returns float64 [sum t*h*w, C*tp*p*p]."""
    rows = []
    for px, (t, h, w) in zip(items, np.asarray(grid_thw, dtype=np.int64).reshape(-1, 3)):
        px = np.asarray(px)
        c, tt = px.shape[:2]
        assert tt == t * temporal_patch, "frames of an item = t * temporal_patch"
        ho, wo = int(h) * patch, int(w) * patch
        sized = np.empty((c, tt, ho, wo), dtype=F64)
        for ci in range(c):
            for fi in range(tt):
                sized[ci, fi] = resize_bilinear(px[ci, fi], ho, wo)
        rows.append(patch_rows(normalise(sized, mean, std), patch, temporal_patch))
    return np.concatenate(rows, axis=0) if rows else np.zeros((0, 0), dtype=F64)
