"""Seeded synthetic workloads for the Encode stage (V_m = E(I_m); paper section 3.1, Eq. 1).

This module only *generates inputs*: configurations, pixel tensors cut into packed patch
rows, segment / grid metadata, random weights, and rounding of those inputs to the
configuration's storage dtype.  It contains none of the encoder's arithmetic and imports
neither the CPU oracle nor the HIP library, so both sides can be fed from it.

The paper evaluates on image datasets that are not available here (section 4.1); these
generators stand in for them with i.i.d. uniform pixels at the image sizes the five
configurations name.  Every tensor is drawn from ``numpy.random.default_rng([seed, stream,
a, b])`` so any layer's weights can be regenerated without holding the whole model.
"""

from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

# RNG stream ids (second entry of the seed sequence)
_STREAM_PIXELS = 1
_STREAM_WEIGHTS = 2

_GLOBAL_TENSORS = ("patch_w", "patch_b", "final_norm_g", "final_norm_b", "merge_w", "merge_b")
_LAYER_TENSORS = ("norm1_g", "norm1_b", "qkv_w", "qkv_b", "proj_w", "proj_b",
                  "norm2_g", "norm2_b", "fc1_w", "fc1_b", "fc2_w", "fc2_b")


@dataclass(frozen=True)
class EncoderConfig:
    """Static description of one encoder; field names follow the C-ABI config struct."""
    name: str
    dtype: str                 # "f32" | "bf16": storage type of weights, input and output
    num_layers: int
    hidden: int                # D
    num_heads: int             # H
    head_dim: int              # d, H*d == D
    mlp_dim: int               # F
    patch: int
    temporal_patch: int
    norm: str                  # "layernorm" | "rmsnorm"
    rope: str                  # "none" | "2d" | "3d"
    rope_pairs: Tuple[int, int, int]   # rotary pairs given to the (t, h, w) axes
    out_dim: int
    in_channels: int = 3
    norm_eps: float = 1e-6
    act: str = "gelu_erf"      # "gelu_erf" | "gelu_tanh"
    use_bias: bool = True
    rope_base: float = 10000.0
    final_norm: bool = True
    merge: int = 2
    seed: int = 0

    @property
    def patch_dim(self) -> int:
        return self.in_channels * self.temporal_patch * self.patch * self.patch

    def replace(self, **kw) -> "EncoderConfig":
        return dataclasses.replace(self, **kw)


C1 = EncoderConfig(name="C1-tiny-f32", dtype="f32", num_layers=1, hidden=256, num_heads=4,
                   head_dim=64, mlp_dim=1024, patch=14, temporal_patch=1, norm="layernorm",
                   rope="2d", rope_pairs=(0, 16, 16), out_dim=512, seed=0)
C2 = EncoderConfig(name="C2-0.6B-bf16-8x448", dtype="bf16", num_layers=24, hidden=1024,
                   num_heads=16, head_dim=64, mlp_dim=4096, patch=16, temporal_patch=1,
                   norm="rmsnorm", rope="2d", rope_pairs=(0, 16, 16), out_dim=4096, seed=0)
C3 = C2.replace(name="C3-0.6B-bf16-varlen32", seed=1)
C4 = EncoderConfig(name="C4-long-bf16-2688", dtype="bf16", num_layers=27, hidden=1152,
                   num_heads=16, head_dim=72, mlp_dim=4304, patch=16, temporal_patch=1,
                   norm="layernorm", rope="2d", rope_pairs=(0, 18, 18), out_dim=3584, seed=0)
C5 = EncoderConfig(name="C5-video-6B-bf16", dtype="bf16", num_layers=45, hidden=3200,
                   num_heads=25, head_dim=128, mlp_dim=12800, patch=14, temporal_patch=2,
                   norm="rmsnorm", rope="3d", rope_pairs=(16, 24, 24), out_dim=8192, seed=0)

# The six image resolutions of the paper's Table 4_2 (section 4.2; the table prints the encoder
# output as [n, 3584] per resolution), pixels as printed.  n follows round(H/28) * round(W/28) --
# patch 14 and a 2x2 merge -- for five of the six rows; the 640 x 960 row prints 529 where the
# rule gives 782, and the rule is used here.  The paper does not describe the encoder behind the
# table beyond its output width: the workload runs the long-sequence encoder (C4: 27 layers,
# hidden 1152 = 16 x 72, MLP 4304, LayerNorm, 2-D rotary, output width 3584) at patch 14 with a
# temporal patch of 2: a still image enters as a clip of two frames and one temporal slice (t = 1),
# the way encoders that share one patch embedding between images and video take it -- and a patch
# row of 3 * 2 * 14 * 14 = 1176 elements is a multiple of 8, which the bf16 kernels require and
# 3 * 14 * 14 = 588 is not.
T42_SIZES_PX = ((280, 280), (560, 560), (640, 960), (720, 1280), (1080, 1920), (4096, 3112))
T42 = C4.replace(name="T42-table4_2-bf16-patch14", patch=14, temporal_patch=2)


def t42_grid(h_px: int, w_px: int) -> Tuple[int, int, int]:
    """Patch grid of one Table 4_2 image: 2 * round(side / 28) patches of 14 pixels per side."""
    return (1, 2 * int(round(h_px / 28.0)), 2 * int(round(w_px / 28.0)))


# Canonical C3 image sizes in pixels (H, W): 32 draws of multiples of 32 in [224, 1344]
# from default_rng(1).integers(7, 43, (32, 2)) * 32, frozen here so that a change in
# NumPy's bit stream cannot change the workload.
C3_SIZES_PX = (
    (768, 800), (1088, 1312), (256, 384), (1152, 1312), (480, 576), (1216, 704),
    (512, 1152), (512, 672), (960, 832), (320, 224), (1216, 1088), (1184, 832),
    (1152, 576), (736, 1120), (352, 544), (352, 736), (1344, 352), (640, 672),
    (1248, 448), (800, 512), (224, 1088), (288, 544), (768, 768), (352, 1344),
    (1056, 1312), (320, 1056), (544, 832), (1280, 512), (1056, 384), (576, 1312),
    (704, 800), (544, 352))


def grids_for(cfg: EncoderConfig) -> List[Tuple[int, int, int]]:
    """Patch grids (t, h, w) of the items of the named configuration's batch."""
    if cfg.name == C1.name:
        return [(1, 16, 16)]
    if cfg.name == C2.name:
        return [(1, 28, 28)] * 8
    if cfg.name == C3.name:
        return [(1, hp // 16, wp // 16) for hp, wp in C3_SIZES_PX]
    if cfg.name == C4.name:
        return [(1, 168, 168)]
    if cfg.name == C5.name:
        return [(8, 32, 32)] * 4
    if cfg.name == T42.name:
        return [t42_grid(h, w) for h, w in T42_SIZES_PX]
    raise KeyError(cfg.name)


CONFIGS: Dict[str, EncoderConfig] = {"C1": C1, "C2": C2, "C3": C3, "C4": C4, "C5": C5, "T42": T42}


# ------------------------------------------------------------------ dtype rounding

def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float32 array to the storage dtype and return it as float32 again."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "bf16":
        return bf16_bits_to_f32(bf16_bits(a))
    raise ValueError(dtype)


# ------------------------------------------------------------------ metadata

def num_tokens(grids: Sequence[Tuple[int, int, int]]) -> int:
    return int(sum(t * h * w for t, h, w in grids))


def num_merged_tokens(grids: Sequence[Tuple[int, int, int]], merge: int = 2) -> int:
    return int(sum(t * (h // merge) * (w // merge) for t, h, w in grids))


def metadata(grids: Sequence[Tuple[int, int, int]], segments: str = "item"):
    """cu_seqlens (int32 [S+1]) and grid_thw (int32 [items, 3]).

    segments = "item": one attention segment per image / clip;
    segments = "frame": one per temporal slice of each item.
    """
    grid_thw = np.asarray(grids, dtype=np.int32).reshape(-1, 3)
    lens: List[int] = []
    for t, h, w in grids:
        if segments == "item":
            lens.append(t * h * w)
        elif segments == "frame":
            lens.extend([h * w] * t)
        else:
            raise ValueError(segments)
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    return cu, grid_thw


# ------------------------------------------------------------------ pixels -> packed patches

def patchify(pixels: np.ndarray, patch: int, temporal_patch: int) -> np.ndarray:
    """[C, t*tp, h*p, w*p] -> [t*h*w, C*tp*p*p].

    Rows are in raster order over (t, h, w); within a row the element order is
    (channel, temporal offset, row in patch, column in patch).
    """
    c, tt, hh, ww = pixels.shape
    t, h, w = tt // temporal_patch, hh // patch, ww // patch
    x = pixels.reshape(c, t, temporal_patch, h, patch, w, patch)
    x = x.transpose(1, 3, 5, 0, 2, 4, 6)          # t h w c tp ph pw
    return np.ascontiguousarray(x.reshape(t * h * w, c * temporal_patch * patch * patch))


def item_pixels(cfg: EncoderConfig, item: int, grid: Tuple[int, int, int], seed=None) -> np.ndarray:
    """U[0,1) pixels of one image or clip, float32 [C, t*tp, h*p, w*p]."""
    t, h, w = grid
    rng = np.random.default_rng([cfg.seed if seed is None else seed, _STREAM_PIXELS, item, 0])
    return rng.random((cfg.in_channels, t * cfg.temporal_patch, h * cfg.patch, w * cfg.patch),
                      dtype=np.float32)


def item_pixels_u8(cfg: EncoderConfig, item: int, grid: Tuple[int, int, int], src_hw: Tuple[int, int] = None,
                   seed=None) -> np.ndarray:
    """Raw pixels of one image or clip as a camera or decoder hands them over: uint8
    [C, t*tp, Hs, Ws], a smooth seeded pattern (low-frequency waves per channel and frame) plus
    uniform noise, so that neighbouring pixels are correlated as in natural images while every
    byte value occurs.  src_hw defaults to the item's grid size in pixels (no resize needed)."""
    t, h, w = grid
    hs, ws = (h * cfg.patch, w * cfg.patch) if src_hw is None else src_hw
    rng = np.random.default_rng([cfg.seed if seed is None else seed, _STREAM_PIXELS, item, 1])
    frames = t * cfg.temporal_patch
    yy = np.arange(hs, dtype=np.float32)[:, None] / max(hs, 1)
    xx = np.arange(ws, dtype=np.float32)[None, :] / max(ws, 1)
    out = np.empty((cfg.in_channels, frames, hs, ws), dtype=np.uint8)
    for c in range(cfg.in_channels):
        for f in range(frames):
            fy, fx, ph = rng.uniform(0.5, 6.0), rng.uniform(0.5, 6.0), rng.uniform(0, 6.28)
            wave = 0.5 + 0.35 * np.sin(6.2832 * (fy * yy + fx * xx) + ph)
            noise = rng.random((hs, ws), dtype=np.float32) * 0.3 - 0.15
            out[c, f] = np.clip(np.rint((wave + noise) * 255.0), 0, 255).astype(np.uint8)
    return out


def packed_patches(cfg: EncoderConfig, grids: Sequence[Tuple[int, int, int]], seed=None) -> np.ndarray:
    """All items' patch rows packed in item order, rounded to cfg.dtype, float32 [T, Pdim]."""
    rows = [patchify(item_pixels(cfg, i, g, seed), cfg.patch, cfg.temporal_patch)
            for i, g in enumerate(grids)]
    return round_to_dtype(np.concatenate(rows, axis=0), cfg.dtype)


# ------------------------------------------------------------------ weights

def _tensor_shape(cfg: EncoderConfig, name: str) -> Tuple[int, ...]:
    D, F = cfg.hidden, cfg.mlp_dim
    return {
        "patch_w": (D, cfg.patch_dim), "patch_b": (D,),
        "final_norm_g": (D,), "final_norm_b": (D,),
        "merge_w": (cfg.out_dim, cfg.merge * cfg.merge * D), "merge_b": (cfg.out_dim,),
        "norm1_g": (D,), "norm1_b": (D,), "qkv_w": (3 * D, D), "qkv_b": (3 * D,),
        "proj_w": (D, D), "proj_b": (D,), "norm2_g": (D,), "norm2_b": (D,),
        "fc1_w": (F, D), "fc1_b": (F,), "fc2_w": (D, F), "fc2_b": (D,),
    }[name]


def _draw(cfg: EncoderConfig, layer: int, tensor_id: int, name: str, std: float) -> np.ndarray:
    rng = np.random.default_rng([cfg.seed, _STREAM_WEIGHTS, layer + 1, tensor_id])
    a = rng.standard_normal(_tensor_shape(cfg, name), dtype=np.float32) * np.float32(std)
    if name.endswith("_g"):                 # norm gains are centred on one
        a = a + np.float32(1.0)
    return a


def _present(cfg: EncoderConfig, name: str) -> bool:
    if name.startswith("final_norm") and not cfg.final_norm:
        return False
    if name in ("norm1_b", "norm2_b", "final_norm_b"):
        return cfg.norm == "layernorm"      # RMSNorm has no shift
    if name.endswith("_b"):
        return cfg.use_bias
    return True


def global_weights(cfg: EncoderConfig, std: float = 0.02) -> Dict[str, np.ndarray]:
    """patch-embed, final-norm and merger tensors (float32 holding cfg.dtype-rounded values)."""
    out = {}
    for i, name in enumerate(_GLOBAL_TENSORS):
        if _present(cfg, name):
            out[name] = round_to_dtype(_draw(cfg, -1, i, name, std), cfg.dtype)
    return out


def layer_weights(cfg: EncoderConfig, layer: int, std: float = 0.02, q_gain: float = 1.0) -> Dict[str, np.ndarray]:
    """One transformer block's tensors.  Linear weights are [out, in] row-major; the rows of
    qkv_w are ordered Q heads, K heads, V heads.  ``q_gain`` multiplies the Q rows (weight
    and bias) before rounding: a gain of 16 gives sharply peaked attention rows."""
    out = {}
    for i, name in enumerate(_LAYER_TENSORS):
        if not _present(cfg, name):
            continue
        a = _draw(cfg, layer, i, name, std)
        if q_gain != 1.0 and name in ("qkv_w", "qkv_b"):
            a[: cfg.hidden] *= np.float32(q_gain)
        out[name] = round_to_dtype(a, cfg.dtype)
    return out


def all_weights(cfg: EncoderConfig, std: float = 0.02, q_gain: float = 1.0):
    """(global dict, list of per-layer dicts).  Only for configurations that fit in memory."""
    return global_weights(cfg, std), [layer_weights(cfg, l, std, q_gain) for l in range(cfg.num_layers)]
