"""ctypes binding of ``libepd_encode.so`` -- argument marshalling only.

The functions below carry the same names and arguments as the C ABI in
``include/epd_encode.h`` (V_m = E(I_m), paper section 3.1, Eq. 1).  PyTorch is used for
device memory and streams and nothing else: every step of the encoder runs in the HIP
library.  There is no fallback: if the library cannot be loaded, importing this module
raises.
"""

from __future__ import annotations

import ctypes as C
from typing import Dict, Iterable, Optional, Sequence

import numpy as np
import torch

from . import build as _build

EPD_OK, EPD_ERR_INVALID_ARG, EPD_ERR_UNSUPPORTED, EPD_ERR_SHAPE, EPD_ERR_WORKSPACE, EPD_ERR_HIP = 0, -1, -2, -3, -4, -5
EPD_F32, EPD_BF16 = 0, 1
EPD_LAYERNORM, EPD_RMSNORM = 0, 1
EPD_GELU_ERF, EPD_GELU_TANH = 0, 1
EPD_ROPE_NONE, EPD_ROPE_2D, EPD_ROPE_3D = 0, 2, 3
(EPD_STEP_PLAN, EPD_STEP_PATCH_EMBED, EPD_STEP_NORM, EPD_STEP_QKV, EPD_STEP_ATTN, EPD_STEP_PROJ,
 EPD_STEP_FC1, EPD_STEP_FC2, EPD_STEP_MERGE, EPD_STEP_COUNT) = range(10)
STEP_NAMES = ["plan", "patch_embed", "norm", "qkv", "attn", "proj", "fc1", "fc2", "merge"]

_LAYER_FIELDS = ["norm1_g", "norm1_b", "qkv_w", "qkv_b", "proj_w", "proj_b",
                 "norm2_g", "norm2_b", "fc1_w", "fc1_b", "fc2_w", "fc2_b"]


class epd_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_FIELDS]


class epd_weights(C.Structure):
    _fields_ = [("patch_w", C.c_void_p), ("patch_b", C.c_void_p),
                ("layers", C.POINTER(epd_layer_weights)),
                ("final_norm_g", C.c_void_p), ("final_norm_b", C.c_void_p),
                ("merge_w", C.c_void_p), ("merge_b", C.c_void_p)]


class epd_encode_cfg(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("dtype", C.c_int32), ("num_layers", C.c_int32),
                ("hidden", C.c_int32), ("num_heads", C.c_int32), ("head_dim", C.c_int32),
                ("mlp_dim", C.c_int32), ("in_channels", C.c_int32), ("patch", C.c_int32),
                ("temporal_patch", C.c_int32), ("norm", C.c_int32), ("norm_eps", C.c_float),
                ("act", C.c_int32), ("use_bias", C.c_int32), ("rope", C.c_int32),
                ("rope_base", C.c_float), ("rope_pairs", C.c_int32 * 3), ("final_norm", C.c_int32),
                ("merge", C.c_int32), ("out_dim", C.c_int32), ("max_tokens", C.c_int32),
                ("max_segments", C.c_int32), ("max_items", C.c_int32),
                ("weights", C.POINTER(epd_weights)), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_uint64)]


EXPORTS = ["epd_encode_workspace_bytes", "epd_encode_create", "epd_encode", "epd_encode_destroy",
           "epd_encode_last_error", "epd_encode_debug_hidden", "epd_encode_set_timing",
           "epd_encode_get_timing", "epd_preprocess"]


def _load() -> C.CDLL:
    lib = C.CDLL(_build.library_path())
    lib.epd_encode_workspace_bytes.restype = C.c_uint64
    lib.epd_encode_workspace_bytes.argtypes = [C.POINTER(epd_encode_cfg)]
    lib.epd_encode_create.restype = C.c_int
    lib.epd_encode_create.argtypes = [C.POINTER(epd_encode_cfg), C.POINTER(C.c_void_p)]
    lib.epd_encode.restype = C.c_int
    lib.epd_encode.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_int32,
                               C.POINTER(C.c_int32), C.c_int32, C.c_void_p, C.c_void_p]
    lib.epd_encode_destroy.restype = C.c_int
    lib.epd_encode_destroy.argtypes = [C.c_void_p]
    lib.epd_preprocess.restype = C.c_int
    lib.epd_preprocess.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32,
                                   C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    lib.epd_encode_last_error.restype = C.c_char_p
    lib.epd_encode_last_error.argtypes = [C.c_void_p]
    lib.epd_encode_debug_hidden.restype = C.c_int
    lib.epd_encode_debug_hidden.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.epd_encode_set_timing.restype = C.c_int
    lib.epd_encode_set_timing.argtypes = [C.c_void_p, C.c_int32]
    lib.epd_encode_get_timing.restype = C.c_int
    lib.epd_encode_get_timing.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                          C.POINTER(C.c_double)]
    return lib


lib = _load()


class EpdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("epd status %d: %s" % (status, message))
        self.status = status


# ---------------------------------------------------------------- same-name wrappers

def epd_encode_workspace_bytes(cfg: epd_encode_cfg) -> int:
    return int(lib.epd_encode_workspace_bytes(C.byref(cfg)))


def epd_encode_last_error(handle: Optional[int]) -> str:
    return lib.epd_encode_last_error(handle).decode()


def epd_encode_create(cfg: epd_encode_cfg) -> int:
    h = C.c_void_p()
    st = lib.epd_encode_create(C.byref(cfg), C.byref(h))
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(None))
    return h.value


def epd_encode(handle, packed_patches: int, cu_seqlens: np.ndarray, grid_thw: np.ndarray,
               out_visual_tokens: int, stream: int) -> None:
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    grid = np.ascontiguousarray(grid_thw, dtype=np.int32).reshape(-1, 3)
    st = lib.epd_encode(handle, packed_patches, cu.ctypes.data_as(C.POINTER(C.c_int32)), len(cu) - 1,
                        grid.ctypes.data_as(C.POINTER(C.c_int32)), grid.shape[0], out_visual_tokens, stream)
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(handle))


def epd_preprocess(handle, pixels: int, src_hw: np.ndarray, grid_thw: np.ndarray, mean, std,
                   packed_patches: int, stream: int) -> None:
    src = np.ascontiguousarray(src_hw, dtype=np.int32).reshape(-1, 2)
    grid = np.ascontiguousarray(grid_thw, dtype=np.int32).reshape(-1, 3)
    mu = np.ascontiguousarray(mean, dtype=np.float32)
    sd = np.ascontiguousarray(std, dtype=np.float32)
    st = lib.epd_preprocess(handle, pixels, src.ctypes.data_as(C.POINTER(C.c_int32)),
                            grid.ctypes.data_as(C.POINTER(C.c_int32)), grid.shape[0],
                            mu.ctypes.data_as(C.POINTER(C.c_float)), sd.ctypes.data_as(C.POINTER(C.c_float)),
                            packed_patches, stream)
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(handle))


def epd_encode_destroy(handle) -> None:
    lib.epd_encode_destroy(handle)


def epd_encode_debug_hidden(handle, out_ptr: int, stream: int) -> None:
    st = lib.epd_encode_debug_hidden(handle, out_ptr, stream)
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(handle))


def epd_encode_set_timing(handle, step: int) -> None:
    st = lib.epd_encode_set_timing(handle, step)
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(handle))


def epd_encode_get_timing(handle):
    ms, n, work = C.c_double(), C.c_int64(), C.c_double()
    st = lib.epd_encode_get_timing(handle, C.byref(ms), C.byref(n), C.byref(work))
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(handle))
    return ms.value, n.value, work.value


# ---------------------------------------------------------------- config marshalling

def make_cfg(cfg, max_tokens: int, max_segments: int, max_items: int) -> epd_encode_cfg:
    """Fill the C config struct from an object with the attribute names of
    ``workloads.EncoderConfig`` (shape fields only; weights / workspace are left empty)."""
    c = epd_encode_cfg()
    c.struct_size = C.sizeof(epd_encode_cfg)
    c.dtype = {"f32": EPD_F32, "bf16": EPD_BF16}[cfg.dtype]
    c.num_layers, c.hidden, c.num_heads, c.head_dim = cfg.num_layers, cfg.hidden, cfg.num_heads, cfg.head_dim
    c.mlp_dim, c.in_channels, c.patch, c.temporal_patch = cfg.mlp_dim, cfg.in_channels, cfg.patch, cfg.temporal_patch
    c.norm = {"layernorm": EPD_LAYERNORM, "rmsnorm": EPD_RMSNORM}[cfg.norm]
    c.norm_eps = cfg.norm_eps
    c.act = {"gelu_erf": EPD_GELU_ERF, "gelu_tanh": EPD_GELU_TANH}[cfg.act]
    c.use_bias = 1 if cfg.use_bias else 0
    c.rope = {"none": EPD_ROPE_NONE, "2d": EPD_ROPE_2D, "3d": EPD_ROPE_3D}[cfg.rope]
    c.rope_base = cfg.rope_base
    c.rope_pairs = (C.c_int32 * 3)(*cfg.rope_pairs)
    c.final_norm = 1 if cfg.final_norm else 0
    c.merge, c.out_dim = cfg.merge, cfg.out_dim
    c.max_tokens, c.max_segments, c.max_items = max_tokens, max_segments, max_items
    return c


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


class EpdEncoder:
    """Owns the device tensors (weights during create, the workspace) and the handle."""

    def __init__(self, cfg, global_weights: Dict[str, np.ndarray], layers: Iterable[Dict[str, np.ndarray]],
                 max_tokens: int, max_segments: int = 64, max_items: int = 64, device: str = "cuda:0"):
        self.cfg = cfg
        self.device = torch.device(device)
        self.dtype = torch_dtype(cfg.dtype)
        self.handle = None
        ccfg = make_cfg(cfg, max_tokens, max_segments, max_items)
        need = epd_encode_workspace_bytes(ccfg)
        if need == 0:
            # let create produce the precise message
            ccfg.weights = C.pointer(epd_weights())
            ccfg.workspace = 256
            epd_encode_create(ccfg)
            raise EpdError(EPD_ERR_INVALID_ARG, "invalid configuration")
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.device).to(self.dtype).contiguous()
        gw = {k: up(v) for k, v in global_weights.items()}
        lws = [{k: up(v) for k, v in lw.items()} for lw in layers]
        if len(lws) != cfg.num_layers:
            raise ValueError("expected %d layers, got %d" % (cfg.num_layers, len(lws)))
        ptr = lambda d, k: d[k].data_ptr() if k in d else None
        arr = (epd_layer_weights * max(1, len(lws)))()
        for i, lw in enumerate(lws):
            for f in _LAYER_FIELDS:
                setattr(arr[i], f, ptr(lw, f))
        w = epd_weights()
        w.patch_w, w.patch_b = ptr(gw, "patch_w"), ptr(gw, "patch_b")
        w.layers = C.cast(arr, C.POINTER(epd_layer_weights))
        w.final_norm_g, w.final_norm_b = ptr(gw, "final_norm_g"), ptr(gw, "final_norm_b")
        w.merge_w, w.merge_b = ptr(gw, "merge_w"), ptr(gw, "merge_b")
        self.workspace = torch.empty(need + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        ccfg.weights = C.pointer(w)
        ccfg.workspace = base
        ccfg.workspace_bytes = need
        self.workspace_bytes = need
        torch.cuda.synchronize(self.device)
        with torch.cuda.device(self.device):
            self.handle = epd_encode_create(ccfg)
        del gw, lws   # the library holds its own copy inside the workspace

    def encode(self, patches: torch.Tensor, cu_seqlens, grid_thw, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """patches: device tensor [T, Pdim] of the configuration's dtype."""
        assert patches.is_cuda and patches.dtype == self.dtype and patches.is_contiguous()
        grid = np.ascontiguousarray(grid_thw, dtype=np.int32).reshape(-1, 3)
        m = self.cfg.merge
        tm = int(sum(int(t) * (int(h) // m) * (int(w) // m) for t, h, w in grid))
        if out is None:
            out = torch.empty((tm, self.cfg.out_dim), dtype=self.dtype, device=self.device)
        assert out.is_cuda and out.dtype == self.dtype and out.is_contiguous() and out.numel() >= tm * self.cfg.out_dim
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            epd_encode(self.handle, patches.data_ptr(), cu_seqlens, grid, out.data_ptr(), stream)
        self._last_T = int(patches.shape[0])
        return out

    def preprocess(self, pixels: torch.Tensor, src_hw, grid_thw, mean, std,
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """pixels: device uint8 tensor, items packed in order, each planar [C, t*tp, Hs, Ws].
        Returns the packed patch rows [T, Pdim] that ``encode`` takes."""
        assert pixels.is_cuda and pixels.dtype == torch.uint8 and pixels.is_contiguous()
        grid = np.ascontiguousarray(grid_thw, dtype=np.int32).reshape(-1, 3)
        src = np.ascontiguousarray(src_hw, dtype=np.int32).reshape(-1, 2)
        assert len(src) == len(grid) and len(mean) == len(std) == self.cfg.in_channels
        need = int(sum(self.cfg.in_channels * int(t) * self.cfg.temporal_patch * int(hs) * int(ws)
                       for (t, _, _), (hs, ws) in zip(grid, src)))
        assert pixels.numel() >= need, "pixel buffer shorter than the items described"
        T = int(sum(int(t) * int(h) * int(w) for t, h, w in grid))
        if out is None:
            out = torch.empty((T, self.cfg.patch_dim), dtype=self.dtype, device=self.device)
        assert out.is_cuda and out.dtype == self.dtype and out.is_contiguous() and out.numel() >= T * self.cfg.patch_dim
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            epd_preprocess(self.handle, pixels.data_ptr(), src, grid, mean, std, out.data_ptr(), stream)
        return out

    def hidden(self) -> torch.Tensor:
        """fp32 residual stream [T, D] of the last call (before the final norm)."""
        out = torch.empty((self._last_T, self.cfg.hidden), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            epd_encode_debug_hidden(self.handle, out.data_ptr(), torch.cuda.current_stream(self.device).cuda_stream)
        return out

    def set_timing(self, step: int) -> None:
        epd_encode_set_timing(self.handle, step)

    def get_timing(self):
        return epd_encode_get_timing(self.handle)

    def close(self) -> None:
        if self.handle is not None:
            torch.cuda.synchronize(self.device)
            epd_encode_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def to_device_patches(patches_f32: np.ndarray, dtype: str, device: str = "cuda:0") -> torch.Tensor:
    """Host float32 rows (already rounded to ``dtype``) -> device tensor of that dtype."""
    return torch.from_numpy(np.ascontiguousarray(patches_f32)).to(device).to(torch_dtype(dtype)).contiguous()
