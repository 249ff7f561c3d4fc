"""Scalar brute-force evaluation of the Encode stage (paper section 3.1, Eq. 1) for tiny inputs.

TEST INFRASTRUCTURE ONLY.  A second, independently written path used to pin
oracle/vit_encode.py: every output element is produced by explicit Python loops over
plain floats (IEEE double) with the ``math`` module -- no NumPy arithmetic, no matrix
routine, no shared helper.  Cost grows as T^2 * D in interpreted code, so callers keep
T <= ~48 and D <= ~32.

Index conventions are restated here on purpose (not imported):
  * token order: items in order, raster over (t, h, w) inside an item;
  * rotary: pair p = elements (p, p + d/2); pairs are dealt to the axes t, h, w in that
    order; j-th pair of an axis with n pairs turns by coord * base**(-j/n);
  * attention: a query attends to the keys of its own segment only, scale 1/sqrt(d);
  * merge: window rows then columns, concatenated, then one linear map.
"""

from __future__ import annotations

import math


def _dot(a, b):
    s = 0.0
    for x, y in zip(a, b):
        s += x * y
    return s


def _affine(x, w, b):
    """x: list[in]; w: list[out][in]; b: list[out] or None."""
    return [_dot(x, w[o]) + (b[o] if b is not None else 0.0) for o in range(len(w))]


def _norm(cfg, x, g, b):
    n = len(x)
    if cfg.norm == "layernorm":
        mu = sum(x) / n
        var = sum((v - mu) * (v - mu) for v in x) / n
        r = 1.0 / math.sqrt(var + cfg.norm_eps)
        return [(x[i] - mu) * r * g[i] + (b[i] if b is not None else 0.0) for i in range(n)]
    ms = sum(v * v for v in x) / n
    r = 1.0 / math.sqrt(ms + cfg.norm_eps)
    return [x[i] * r * g[i] for i in range(n)]


def _act(cfg, v):
    if cfg.act == "gelu_erf":
        return 0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0)))
    return 0.5 * v * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (v + 0.044715 * v * v * v)))


def _coords(grid_thw):
    out = []
    for (t, h, w) in grid_thw:
        for ti in range(t):
            for r in range(h):
                for c in range(w):
                    out.append((ti, r, c))
    return out


def _rotate(cfg, vec, coord):
    """vec: one head vector (list[d]); returns the rotated copy."""
    d = len(vec)
    half = d // 2
    out = list(vec)
    p = 0
    for axis in range(3):
        n = cfg.rope_pairs[axis]
        for j in range(n):
            ang = coord[axis] * cfg.rope_base ** (-float(j) / n)
            c, s = math.cos(ang), math.sin(ang)
            a, b = vec[p], vec[p + half]
            out[p] = a * c - b * s
            out[p + half] = a * s + b * c
            p += 1
    assert p == half or cfg.rope == "none"
    return out


def attention(q, k, v, cu_seqlens):
    """q, k, v: nested lists [T][H][d] -> [T][H][d]; plain definition, one element at a time."""
    T, H, d = len(q), len(q[0]), len(q[0][0])
    out = [[[0.0] * d for _ in range(H)] for _ in range(T)]
    for s in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        for i in range(lo, hi):
            for h in range(H):
                sc = [_dot(q[i][h], k[j][h]) / math.sqrt(d) for j in range(lo, hi)]
                m = max(sc)
                e = [math.exp(x - m) for x in sc]
                z = sum(e)
                for c in range(d):
                    acc = 0.0
                    for jj, j in enumerate(range(lo, hi)):
                        acc += e[jj] / z * v[j][h][c]
                    out[i][h][c] = acc
    return out


def encode(cfg, gw, layers, patches, cu_seqlens, grid_thw, coord_offset=(0, 0, 0)):
    """Same contract as oracle.vit_encode.encode, inputs as nested lists (or anything
    indexable that yields Python floats via float())."""
    tolist = lambda a: None if a is None else [[float(v) for v in row] for row in a]
    tovec = lambda a: None if a is None else [float(v) for v in a]
    H, d = cfg.num_heads, cfg.head_dim
    D = H * d
    grid = [tuple(int(v) for v in g) for g in grid_thw]
    coords = [(c[0] + coord_offset[0], c[1] + coord_offset[1], c[2] + coord_offset[2])
              for c in _coords(grid)]
    pw, pb = tolist(gw["patch_w"]), tovec(gw.get("patch_b"))
    x = [_affine([float(v) for v in row], pw, pb) for row in patches]
    T = len(x)
    assert T == len(coords)
    for lw in layers:
        qkv_w, qkv_b = tolist(lw["qkv_w"]), tovec(lw.get("qkv_b"))
        n1g, n1b = tovec(lw["norm1_g"]), tovec(lw.get("norm1_b"))
        q = [[None] * H for _ in range(T)]
        k = [[None] * H for _ in range(T)]
        v = [[None] * H for _ in range(T)]
        for i in range(T):
            row = _affine(_norm(cfg, x[i], n1g, n1b), qkv_w, qkv_b)
            for h in range(H):
                qh = row[h * d:(h + 1) * d]
                kh = row[D + h * d:D + (h + 1) * d]
                vh = row[2 * D + h * d:2 * D + (h + 1) * d]
                if cfg.rope != "none":
                    qh, kh = _rotate(cfg, qh, coords[i]), _rotate(cfg, kh, coords[i])
                q[i][h], k[i][h], v[i][h] = qh, kh, vh
        o = attention(q, k, v, cu_seqlens)
        proj_w, proj_b = tolist(lw["proj_w"]), tovec(lw.get("proj_b"))
        n2g, n2b = tovec(lw["norm2_g"]), tovec(lw.get("norm2_b"))
        f1w, f1b = tolist(lw["fc1_w"]), tovec(lw.get("fc1_b"))
        f2w, f2b = tolist(lw["fc2_w"]), tovec(lw.get("fc2_b"))
        for i in range(T):
            flat = [o[i][h][c] for h in range(H) for c in range(d)]
            upd = _affine(flat, proj_w, proj_b)
            x[i] = [x[i][c] + upd[c] for c in range(D)]
            hid = [_act(cfg, u) for u in _affine(_norm(cfg, x[i], n2g, n2b), f1w, f1b)]
            upd = _affine(hid, f2w, f2b)
            x[i] = [x[i][c] + upd[c] for c in range(D)]
    if cfg.final_norm:
        fg, fb = tovec(gw["final_norm_g"]), tovec(gw.get("final_norm_b"))
        x = [_norm(cfg, row, fg, fb) for row in x]
    mw, mb = tolist(gw["merge_w"]), tovec(gw.get("merge_b"))
    m = cfg.merge
    out = []
    base = 0
    for (t, h, w) in grid:
        for ti in range(t):
            for i in range(h // m):
                for j in range(w // m):
                    cat = []
                    for di in range(m):
                        for dj in range(m):
                            cat.extend(x[base + (ti * h + m * i + di) * w + m * j + dj])
                    out.append(_affine(cat, mw, mb))
        base += t * h * w
    return out
