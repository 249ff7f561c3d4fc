"""CPU oracle of the Encode stage, V_m = E(I_m) with V_m in R^{n x d} (paper section 3.1, Eq. 1).

TEST INFRASTRUCTURE ONLY.  This file defines what "correct" means for the HIP library and
is imported only by the tests, the smoke check and the bench's CPU-baseline leg.  It shares
no code with the HIP path and imports nothing from the package.

The paper fixes the contract (multimodal input in, one d-dimensional row per visual token
out) but not the encoder's internals; the encoder evaluated here is the plain pre-norm
Vision Transformer the five benchmark configurations describe, written out definition by
definition in float64 NumPy:

  tokens -> patch embedding -> L x [norm, QKV, rotary, per-segment softmax attention,
  output projection + residual, norm, GELU MLP + residual] -> final norm -> 2x2 spatial
  merge -> projection.

Nothing is blocked, fused or reordered except that attention rows are processed in slabs of
query rows to bound memory (each softmax row is still formed in full).

Pins (tests/test_oracle_*.py): scalar brute force (oracle/brute_force.py), softmax row sums,
segment isolation, permutation equivariance, rotary relative-position property, norm
moments, GELU closed-form values, L = 0 closed form (two matmuls), and the merged-token
counts printed in the paper's Table 4_2.  End-to-end output *values* are not printed
anywhere in the paper: end-to-end parity is pinned only through those parts and through the
agreement of the two independently written paths.

``cfg`` is any object with the attributes: num_layers, hidden, num_heads, head_dim, mlp_dim,
norm ("layernorm" | "rmsnorm"), norm_eps, act ("gelu_erf" | "gelu_tanh"), rope ("none" |
"2d" | "3d"), rope_pairs (nt, nh, nw), rope_base, final_norm, merge.
"""

from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# ----------------------------------------------------------------------------- tokens

def token_coords(grid_thw) -> np.ndarray:
    """Per-token coordinates (ti, row, col), int64 [T, 3].

    Items are packed in order; item (t, h, w) contributes t*h*w tokens in raster order,
    token index (ti*h + r)*w + c, each coordinate starting at 0 in every item.
    """
    out = []
    for t, h, w in np.asarray(grid_thw, dtype=np.int64).reshape(-1, 3):
        ti, r, c = np.meshgrid(np.arange(t), np.arange(h), np.arange(w), indexing="ij")
        out.append(np.stack([ti.ravel(), r.ravel(), c.ravel()], axis=1))
    return np.concatenate(out, axis=0) if out else np.zeros((0, 3), dtype=np.int64)


def merged_token_count(grid_thw, merge: int = 2) -> int:
    """n of Eq. 1 after the spatial merge: sum over items of t * (h/merge) * (w/merge)."""
    g = np.asarray(grid_thw, dtype=np.int64).reshape(-1, 3)
    return int(np.sum(g[:, 0] * (g[:, 1] // merge) * (g[:, 2] // merge)))


# ----------------------------------------------------------------------------- pointwise parts

def layer_norm(x, gamma, beta, eps):
    """(x - mean) / sqrt(var + eps) * gamma + beta, biased variance over the last axis."""
    x = np.asarray(x, F64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    y = (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, F64)
    return y if beta is None else y + np.asarray(beta, F64)


def rms_norm(x, gamma, eps):
    """x / sqrt(mean(x^2) + eps) * gamma over the last axis."""
    x = np.asarray(x, F64)
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gamma, F64)


def norm(cfg, x, gamma, beta):
    if cfg.norm == "layernorm":
        return layer_norm(x, gamma, beta, cfg.norm_eps)
    if cfg.norm == "rmsnorm":
        return rms_norm(x, gamma, cfg.norm_eps)
    raise ValueError(cfg.norm)


def gelu_erf(x):
    """x * Phi(x) with the exact Gaussian CDF."""
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + _erf(x / np.sqrt(2.0)))


def gelu_tanh(x):
    x = np.asarray(x, F64)
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def activation(cfg, x):
    return gelu_erf(x) if cfg.act == "gelu_erf" else gelu_tanh(x)


def linear(x, w, b):
    """x @ w^T + b with w stored [out, in]."""
    y = np.asarray(x, F64) @ np.asarray(w, F64).T
    return y if b is None else y + np.asarray(b, F64)


# ----------------------------------------------------------------------------- rotary

def rotary_angles(coords, rope_pairs, base) -> np.ndarray:
    """Angles theta[T, d/2].

    The d/2 rotation pairs are handed to the axes in the order t, h (row), w (column);
    the j-th pair of an axis with n pairs turns by coordinate * base^(-j/n).
    """
    coords = np.asarray(coords, F64)
    cols = []
    for axis, n in enumerate(rope_pairs):
        if n == 0:
            continue
        freq = float(base) ** (-np.arange(n, dtype=F64) / n)
        cols.append(coords[:, axis:axis + 1] * freq[None, :])
    return np.concatenate(cols, axis=1) if cols else np.zeros((coords.shape[0], 0), F64)


def apply_rotary(x, theta):
    """Rotate x[T, H, d]; pair p is made of elements (p, p + d/2) of each head vector."""
    x = np.asarray(x, F64)
    half = x.shape[-1] // 2
    assert theta.shape == (x.shape[0], half)
    cos, sin = np.cos(theta)[:, None, :], np.sin(theta)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * cos - hi * sin, lo * sin + hi * cos], axis=-1)


# ----------------------------------------------------------------------------- attention

def softmax_rows(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def attention_varlen(q, k, v, cu_seqlens, slab: int = 2048, return_probs: bool = False):
    """Block-diagonal, non-causal softmax(Q K^T / sqrt(d)) V.

    q, k, v: [T, H, d]; segment s is the token range [cu[s], cu[s+1]); a query sees exactly
    the keys of its own segment.  Returns [T, H, d] (and the list of per-segment
    probability tensors [H, n, n] when return_probs).
    """
    q, k, v = (np.asarray(a, F64) for a in (q, k, v))
    T, H, d = q.shape
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    out = np.zeros_like(q)
    probs = []
    scale = 1.0 / np.sqrt(float(d))
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        seg_p = []
        for h in range(H):
            kh, vh = k[a:b, h, :], v[a:b, h, :]
            rows = []
            for r0 in range(a, b, slab):
                r1 = min(b, r0 + slab)
                p = softmax_rows((q[r0:r1, h, :] @ kh.T) * scale)
                out[r0:r1, h, :] = p @ vh
                if return_probs:
                    rows.append(p)
            if return_probs:
                seg_p.append(np.concatenate(rows, axis=0))
        if return_probs:
            probs.append(np.stack(seg_p, axis=0))
    return (out, probs) if return_probs else out


# ----------------------------------------------------------------------------- merger

def merge_gather_index(grid_thw, merge: int = 2) -> np.ndarray:
    """Source token of every slot of every merged token, int64 [Tm, merge*merge].

    Merged token (ti, i, j) of an item, raster order over (t, h/m, w/m), gathers the
    window rows 0..m-1 and columns 0..m-1 in row-major order: for m = 2 the sources are
    (2i,2j), (2i,2j+1), (2i+1,2j), (2i+1,2j+1).
    """
    idx = []
    base = 0
    for t, h, w in np.asarray(grid_thw, dtype=np.int64).reshape(-1, 3):
        assert h % merge == 0 and w % merge == 0
        for ti in range(t):
            for i in range(h // merge):
                for j in range(w // merge):
                    idx.append([base + (ti * h + merge * i + di) * w + merge * j + dj
                                for di in range(merge) for dj in range(merge)])
        base += t * h * w
    return np.asarray(idx, dtype=np.int64).reshape(-1, merge * merge)


def merge_tokens(z, grid_thw, merge: int = 2):
    """[T, D] -> [Tm, merge*merge*D]: concatenation of each window's rows."""
    z = np.asarray(z, F64)
    idx = merge_gather_index(grid_thw, merge)
    return z[idx].reshape(idx.shape[0], -1)


# ----------------------------------------------------------------------------- whole encoder

def encoder_layer(cfg, x, lw, theta, cu_seqlens):
    """One pre-norm block: x + Attn(norm(x)), then x + MLP(norm(x))."""
    T = x.shape[0]
    H, d = cfg.num_heads, cfg.head_dim
    a = norm(cfg, x, lw["norm1_g"], lw.get("norm1_b"))
    qkv = linear(a, lw["qkv_w"], lw.get("qkv_b"))
    q = qkv[:, 0 * H * d:1 * H * d].reshape(T, H, d)
    k = qkv[:, 1 * H * d:2 * H * d].reshape(T, H, d)
    v = qkv[:, 2 * H * d:3 * H * d].reshape(T, H, d)
    if theta is not None:
        q, k = apply_rotary(q, theta), apply_rotary(k, theta)
    o = attention_varlen(q, k, v, cu_seqlens).reshape(T, H * d)
    x = x + linear(o, lw["proj_w"], lw.get("proj_b"))
    b = norm(cfg, x, lw["norm2_g"], lw.get("norm2_b"))
    hdn = activation(cfg, linear(b, lw["fc1_w"], lw.get("fc1_b")))
    return x + linear(hdn, lw["fc2_w"], lw.get("fc2_b"))


def encode(cfg, gw, layers, patches, cu_seqlens, grid_thw, *, coord_offset=None,
           return_hidden: bool = False):
    """V_m = E(I_m): packed patch rows [T, Pdim] -> visual tokens [Tm, out_dim], float64.

    gw: dict with patch_w, patch_b, final_norm_g(, final_norm_b), merge_w, merge_b.
    layers: sequence (or generator) of per-layer dicts, consumed one at a time.
    coord_offset: optional (dt, dh, dw) added to every rotary coordinate (test hook).
    return_hidden: also return the residual stream [T, D] before the final norm.
    """
    x = linear(patches, gw["patch_w"], gw.get("patch_b"))
    theta = None
    if cfg.rope != "none":
        coords = token_coords(grid_thw)
        if coord_offset is not None:
            coords = coords + np.asarray(coord_offset, dtype=np.int64)[None, :]
        theta = rotary_angles(coords, cfg.rope_pairs, cfg.rope_base)
    n_done = 0
    for lw in layers:
        x = encoder_layer(cfg, x, lw, theta, cu_seqlens)
        n_done += 1
    assert n_done == cfg.num_layers, (n_done, cfg.num_layers)
    hidden = x
    z = norm(cfg, x, gw["final_norm_g"], gw.get("final_norm_b")) if cfg.final_norm else x
    g = merge_tokens(z, grid_thw, cfg.merge) if cfg.merge > 1 else z
    y = linear(g, gw["merge_w"], gw.get("merge_b"))
    return (y, hidden) if return_hidden else y
