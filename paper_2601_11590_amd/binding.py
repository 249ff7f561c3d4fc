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
EPD_MISS = 1
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
           "epd_encode_last_error", "epd_encode_debug_hidden", "epd_encode_set_timing", "epd_encode_set_tuning", "epd_encode_set_compute_units",
           "epd_encode_get_timing", "epd_preprocess", "epd_encode_cached", "epd_store_create",
           "epd_store_destroy", "epd_store_last_error", "epd_store_hash", "epd_store_hash_noalloc", "epd_store_lookup", "epd_store_insert",
           "epd_store_stats", "epd_probe_stream_read", "epd_probe_mfma_rate", "epd_probe_gemm_plan"]


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
    U64P, I32P, F32P = C.POINTER(C.c_uint64), C.POINTER(C.c_int32), C.POINTER(C.c_float)
    lib.epd_store_create.restype = C.c_int
    lib.epd_store_create.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(C.c_void_p)]
    lib.epd_store_destroy.restype = C.c_int
    lib.epd_store_destroy.argtypes = [C.c_void_p]
    lib.epd_store_last_error.restype = C.c_char_p
    lib.epd_store_last_error.argtypes = [C.c_void_p]
    lib.epd_store_hash.restype = C.c_int
    lib.epd_store_hash.argtypes = [C.c_void_p, C.c_void_p, U64P, U64P, C.c_int32, U64P, C.c_void_p]
    lib.epd_store_hash_noalloc.restype = C.c_int
    lib.epd_store_hash_noalloc.argtypes = [C.c_void_p, U64P, U64P, C.c_int32, C.c_void_p, C.c_void_p]
    lib.epd_store_lookup.restype = C.c_int
    lib.epd_store_lookup.argtypes = [C.c_void_p, U64P, C.POINTER(C.c_void_p), U64P]
    lib.epd_store_insert.restype = C.c_int
    lib.epd_store_insert.argtypes = [C.c_void_p, U64P, C.c_uint64, C.POINTER(C.c_void_p)]
    lib.epd_store_stats.restype = C.c_int
    lib.epd_store_stats.argtypes = [C.c_void_p, U64P, U64P, U64P, U64P]
    lib.epd_encode_cached.restype = C.c_int
    lib.epd_encode_cached.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, I32P, I32P, C.c_int32, F32P, F32P,
                                      C.c_void_p, C.c_void_p, C.c_void_p, I32P, U64P, C.c_void_p]
    lib.epd_preprocess.restype = C.c_int
    lib.epd_preprocess.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32,
                                   C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
    lib.epd_encode_last_error.restype = C.c_char_p
    lib.epd_encode_last_error.argtypes = [C.c_void_p]
    lib.epd_encode_debug_hidden.restype = C.c_int
    lib.epd_encode_debug_hidden.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.epd_encode_set_timing.restype = C.c_int
    lib.epd_encode_set_timing.argtypes = [C.c_void_p, C.c_int32]
    lib.epd_encode_set_compute_units.restype = C.c_int
    lib.epd_encode_set_compute_units.argtypes = [C.c_void_p, C.c_int32]
    lib.epd_probe_stream_read.restype = C.c_int
    lib.epd_probe_stream_read.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_int32, C.c_void_p]
    lib.epd_probe_mfma_rate.restype = C.c_int
    lib.epd_probe_mfma_rate.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_double), C.c_void_p]
    lib.epd_probe_gemm_plan.restype = C.c_int
    lib.epd_probe_gemm_plan.argtypes = [C.c_int32] * 6 + [C.POINTER(C.c_int32)] * 3
    lib.epd_encode_set_tuning.restype = C.c_int
    lib.epd_encode_set_tuning.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
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


class StoreError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("epd store status %d: %s" % (status, message))
        self.status = status


def epd_store_last_error(store: Optional[int]) -> str:
    return lib.epd_store_last_error(store).decode()


def epd_store_create(pool_ptr: int, pool_bytes: int) -> int:
    s = C.c_void_p()
    st = lib.epd_store_create(pool_ptr, pool_bytes, C.byref(s))
    if st != EPD_OK:
        raise StoreError(st, epd_store_last_error(None))
    return s.value


def epd_store_destroy(store) -> None:
    lib.epd_store_destroy(store)


def _key(key):
    return (C.c_uint64 * 2)(int(key[0]), int(key[1]))


def epd_store_lookup(store, key):
    """(device pointer, bytes) of a stored value, or None."""
    p, n = C.c_void_p(), C.c_uint64()
    st = lib.epd_store_lookup(store, _key(key), C.byref(p), C.byref(n))
    if st == EPD_MISS:
        return None
    if st != EPD_OK:
        raise StoreError(st, epd_store_last_error(store))
    return p.value, n.value


def epd_store_insert(store, key, nbytes: int) -> int:
    p = C.c_void_p()
    st = lib.epd_store_insert(store, _key(key), nbytes, C.byref(p))
    if st != EPD_OK:
        raise StoreError(st, epd_store_last_error(store))
    return p.value


def epd_store_stats(store):
    v = [C.c_uint64() for _ in range(4)]
    st = lib.epd_store_stats(store, *[C.byref(x) for x in v])
    if st != EPD_OK:
        raise StoreError(st, epd_store_last_error(store))
    return dict(zip(("hits", "misses", "evictions", "entries"), (x.value for x in v)))


def epd_store_hash(store, data_ptr: int, offsets, salts, stream: int) -> np.ndarray:
    """uint64 [n, 2] keys of the byte ranges [offsets[i], offsets[i+1]) of one device buffer."""
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    sa = np.ascontiguousarray(salts, dtype=np.uint64)
    n = len(sa)
    assert len(off) == n + 1
    keys = np.zeros((n, 2), dtype=np.uint64)
    U64P = C.POINTER(C.c_uint64)
    st = lib.epd_store_hash(store, data_ptr, off.ctypes.data_as(U64P), sa.ctypes.data_as(U64P), n,
                            keys.ctypes.data_as(U64P), stream)
    if st != EPD_OK:
        raise StoreError(st, epd_store_last_error(store))
    return keys


def epd_store_hash_noalloc(data_ptr: int, offsets, salts, keys_device_ptr: int, stream: int) -> None:
    """Keys of the byte ranges into a device buffer uint64 [n, 2]; enqueues only (no wait)."""
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    sa = np.ascontiguousarray(salts, dtype=np.uint64)
    assert len(off) == len(sa) + 1
    U64P = C.POINTER(C.c_uint64)
    st = lib.epd_store_hash_noalloc(data_ptr, off.ctypes.data_as(U64P), sa.ctypes.data_as(U64P), len(sa), keys_device_ptr, stream)
    if st != EPD_OK:
        raise StoreError(st, epd_store_last_error(None))


def epd_encode_cached(handle, store, model_salt: int, pixels: int, src_hw, grid_thw, mean, std, rows_scratch: int,
                      out_scratch: int, out_visual_tokens: int, stream: int):
    """Returns (hit flags int32 [items], keys uint64 [items, 2])."""
    src = np.ascontiguousarray(src_hw, dtype=np.int32).reshape(-1, 2)
    grid = np.ascontiguousarray(grid_thw, dtype=np.int32).reshape(-1, 3)
    mu = np.ascontiguousarray(mean, dtype=np.float32)
    sd = np.ascontiguousarray(std, dtype=np.float32)
    hit = np.zeros(grid.shape[0], dtype=np.int32)
    keys = np.zeros((grid.shape[0], 2), dtype=np.uint64)
    I32P, F32P, U64P = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_uint64)
    st = lib.epd_encode_cached(handle, store, model_salt, pixels, src.ctypes.data_as(I32P), grid.ctypes.data_as(I32P),
                               grid.shape[0], mu.ctypes.data_as(F32P), sd.ctypes.data_as(F32P), rows_scratch, out_scratch,
                               out_visual_tokens, hit.ctypes.data_as(I32P), keys.ctypes.data_as(U64P), stream)
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(handle))
    return hit, keys


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


def epd_encode_set_tuning(handle, gemm_tile: int, attn_groups: int) -> None:
    st = lib.epd_encode_set_tuning(handle, gemm_tile, attn_groups)
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(handle))


def epd_encode_set_compute_units(handle, compute_units: int) -> None:
    st = lib.epd_encode_set_compute_units(handle, compute_units)
    if st != EPD_OK:
        raise EpdError(st, epd_encode_last_error(handle))


def epd_probe_stream_read(buf_ptr: int, nbytes: int, out_ptr: int, blocks: int, stream: int) -> None:
    st = lib.epd_probe_stream_read(buf_ptr, nbytes, out_ptr, blocks, stream)
    if st != EPD_OK:
        raise EpdError(st, "epd_probe_stream_read: bad argument or launch failure")


def epd_probe_mfma_rate(shape: int, zero_operands: bool, iters: int, out_ptr: int, stream: int) -> float:
    """Enqueue one launch of the matrix-core rate probe; returns the flops it executes."""
    fl = C.c_double()
    st = lib.epd_probe_mfma_rate(shape, 1 if zero_operands else 0, iters, out_ptr, C.byref(fl), stream)
    if st != EPD_OK:
        raise EpdError(st, "epd_probe_mfma_rate: bad argument or launch failure")
    return fl.value


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

    def encode_cached(self, store: "MMStore", model_salt: int, pixels: torch.Tensor, src_hw, grid_thw, mean, std,
                      out: Optional[torch.Tensor] = None):
        """Raw pixels -> visual tokens through the store.  Returns (out, hit flags, keys)."""
        assert pixels.is_cuda and pixels.dtype == torch.uint8 and pixels.is_contiguous()
        grid = np.ascontiguousarray(grid_thw, dtype=np.int32).reshape(-1, 3)
        src = np.ascontiguousarray(src_hw, dtype=np.int32).reshape(-1, 2)
        assert len(src) == len(grid)
        need = int(sum(self.cfg.in_channels * int(t) * self.cfg.temporal_patch * int(hs) * int(ws)
                       for (t, _, _), (hs, ws) in zip(grid, src)))
        assert pixels.numel() >= need, "pixel buffer shorter than the items described"
        m = self.cfg.merge
        T = int(sum(int(t) * int(h) * int(w) for t, h, w in grid))
        tm = int(sum(int(t) * (int(h) // m) * (int(w) // m) for t, h, w in grid))
        rows = torch.empty((max(T, 1), self.cfg.patch_dim), dtype=self.dtype, device=self.device)
        tmp = torch.empty((max(tm, 1), self.cfg.out_dim), dtype=self.dtype, device=self.device)
        if out is None:
            out = torch.empty((tm, self.cfg.out_dim), dtype=self.dtype, device=self.device)
        assert out.is_cuda and out.dtype == self.dtype and out.is_contiguous() and out.numel() >= tm * self.cfg.out_dim
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            hit, keys = epd_encode_cached(self.handle, store.handle, model_salt, pixels.data_ptr(), src, grid, mean, std,
                                          rows.data_ptr(), tmp.data_ptr(), out.data_ptr(), stream)
            # the scratch tensors are read by work queued on this stream: keep them until it is through
            rows.record_stream(torch.cuda.current_stream(self.device))
            tmp.record_stream(torch.cuda.current_stream(self.device))
        return out, hit, keys

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

    def set_tuning(self, gemm_tile: int = -1, attn_groups: int = 0) -> None:
        epd_encode_set_tuning(self.handle, gemm_tile, attn_groups)

    def set_compute_units(self, compute_units: int = 0) -> None:
        epd_encode_set_compute_units(self.handle, compute_units)

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


class MMStore:
    """Device pool + the library's store handle (single-node stand-in for the paper's MM Store)."""

    def __init__(self, pool_bytes: int, device: str = "cuda:0"):
        self.device = torch.device(device)
        self.pool = torch.empty(pool_bytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.pool.data_ptr() + 255) // 256 * 256
        self.base = base
        self.handle = epd_store_create(base, pool_bytes)

    def hash(self, data: torch.Tensor, offsets, salts) -> np.ndarray:
        assert data.is_cuda and data.dtype == torch.uint8 and data.is_contiguous()
        assert int(np.asarray(offsets)[-1]) <= data.numel()
        with torch.cuda.device(self.device):
            return epd_store_hash(self.handle, data.data_ptr(), offsets, salts, torch.cuda.current_stream(self.device).cuda_stream)

    def stats(self):
        return epd_store_stats(self.handle)

    def close(self) -> None:
        if self.handle is not None:
            torch.cuda.synchronize(self.device)
            epd_store_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def to_device_patches(patches_f32: np.ndarray, dtype: str, device: str = "cuda:0") -> torch.Tensor:
    """Host float32 rows (already rounded to ``dtype``) -> device tensor of that dtype."""
    return torch.from_numpy(np.ascontiguousarray(patches_f32)).to(device).to(torch_dtype(dtype)).contiguous()


EPI_STORE, EPI_GELU, EPI_RESIDUAL, EPI_QKV = 0, 1, 2, 3


def epd_probe_gemm_plan(M: int, N: int, K: int, epilogue: int = EPI_STORE, qk_cols: int = 0, compute_units: int = 0):
    """(tile_rows, tile_cols, body_rows) of the layer GEMM's launch plan for an M x N x K product (host only)."""
    tr, tc, br = C.c_int32(), C.c_int32(), C.c_int32()
    st = lib.epd_probe_gemm_plan(M, N, K, epilogue, qk_cols, compute_units, C.byref(tr), C.byref(tc), C.byref(br))
    if st != EPD_OK:
        raise EpdError(st, "epd_probe_gemm_plan: bad argument")
    return tr.value, tc.value, br.value
