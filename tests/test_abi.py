"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, the ctypes mirror of the structs matches the C layout, and every configuration
error is reported on the host before any HIP call (no GPU needed, nothing is launched)."""

import ctypes as C
import os
import re
import subprocess
import sys

import pytest

from paper_2601_11590_amd import binding as B, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "epd_encode.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(epd_(?:encode|preprocess|store|probe)\w*)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS), (names, B.EXPORTS)
    for n in names:
        assert getattr(B.lib, n) is not None


def test_header_compiles_as_plain_c_and_layout_matches_ctypes(tmp_path):
    src = tmp_path / "probe.c"
    fields = [f for f, _ in B.epd_encode_cfg._fields_]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "epd_encode.h"', "int main(void) {",
             'printf("%zu %zu %zu\\n", sizeof(epd_encode_cfg), sizeof(epd_weights), sizeof(epd_layer_weights));']
    for f in fields:
        lines.append('printf("%s %%zu\\n", offsetof(epd_encode_cfg, %s));' % (f, f))
    lines += ["return 0; }"]
    src.write_text("\n".join(lines))
    exe = tmp_path / "probe"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, stdout=subprocess.PIPE, text=True).stdout.split("\n")
    sizes = [int(v) for v in out[0].split()]
    assert sizes == [C.sizeof(B.epd_encode_cfg), C.sizeof(B.epd_weights), C.sizeof(B.epd_layer_weights)]
    for line in out[1:]:
        if line.strip():
            name, off = line.split()
            assert getattr(B.epd_encode_cfg, name).offset == int(off), name


def test_status_and_enum_values_match_header():
    text = open(HEADER).read()
    for name in ["EPD_OK", "EPD_ERR_INVALID_ARG", "EPD_ERR_UNSUPPORTED", "EPD_ERR_SHAPE", "EPD_ERR_WORKSPACE",
                 "EPD_ERR_HIP", "EPD_F32", "EPD_BF16", "EPD_LAYERNORM", "EPD_RMSNORM", "EPD_GELU_ERF", "EPD_GELU_TANH",
                 "EPD_ROPE_NONE", "EPD_ROPE_2D", "EPD_ROPE_3D", "EPD_STEP_PLAN", "EPD_STEP_MERGE", "EPD_STEP_COUNT"]:
        m = re.search(r"\b%s\s*=\s*(-?\d+)" % name, text)
        assert m, name
        assert int(m.group(1)) == getattr(B, name), name


def test_workspace_bytes_is_pure_host_arithmetic():
    for key, cfg in W.CONFIGS.items():
        grids = W.grids_for(cfg)
        c = B.make_cfg(cfg, W.num_tokens(grids), len(grids), len(grids))
        need = B.epd_encode_workspace_bytes(c)
        params = cfg.patch_dim * cfg.hidden + cfg.num_layers * (4 * cfg.hidden ** 2 + 2 * cfg.hidden * cfg.mlp_dim) \
            + 4 * cfg.hidden * cfg.out_dim
        es = 4 if cfg.dtype == "f32" else 2
        assert need > params * es, key                      # at least the weight copy
        assert need < params * es + W.num_tokens(grids) * (cfg.hidden * 24 + cfg.mlp_dim * 4) + (64 << 20), key
    assert B.epd_encode_workspace_bytes(B.make_cfg(W.C2, 6272, 8, 8)) % 256 == 0


def _create_error(cfg_obj, mutate=None, max_tokens=64, with_buffers=True):
    c = B.make_cfg(cfg_obj, max_tokens, 4, 4)
    w = B.epd_weights()
    lw = (B.epd_layer_weights * max(1, cfg_obj.num_layers))()
    if with_buffers:
        for f, _ in B.epd_layer_weights._fields_:
            for l in lw:
                setattr(l, f, 0x1000)
        for f in ("patch_w", "patch_b", "final_norm_g", "final_norm_b", "merge_w", "merge_b"):
            setattr(w, f, 0x1000)
        w.layers = C.cast(lw, C.POINTER(B.epd_layer_weights))
        c.weights = C.pointer(w)
        c.workspace = 0x100000
        c.workspace_bytes = 1 << 40
    if mutate:
        mutate(c)
    h = C.c_void_p()
    st = B.lib.epd_encode_create(C.byref(c), C.byref(h))
    assert not h.value
    return st, B.epd_encode_last_error(None)


TINY = W.EncoderConfig(name="t", dtype="bf16", num_layers=1, hidden=64, num_heads=1, head_dim=64, mlp_dim=128,
                       patch=4, temporal_patch=1, norm="rmsnorm", rope="2d", rope_pairs=(0, 16, 16), out_dim=64)


@pytest.mark.parametrize("change,status,needle", [
    (dict(head_dim=60, num_heads=1), B.EPD_ERR_UNSUPPORTED, "hidden"),
    (dict(rope_pairs=(0, 16, 15)), B.EPD_ERR_UNSUPPORTED, "rope_pairs"),
    (dict(hidden=36, num_heads=1, head_dim=36, rope_pairs=(0, 9, 9)), B.EPD_ERR_UNSUPPORTED, "multiples of 8"),
    (dict(hidden=40, num_heads=1, head_dim=40, rope_pairs=(0, 10, 10)), B.EPD_ERR_UNSUPPORTED, "attention kernel"),
    (dict(mlp_dim=100), B.EPD_ERR_UNSUPPORTED, "multiples of 8"),
    (dict(num_layers=-1), B.EPD_ERR_INVALID_ARG, "non-positive"),
    (dict(merge=0), B.EPD_ERR_INVALID_ARG, "non-positive"),
])
def test_create_rejects_bad_shapes_on_the_host(change, status, needle):
    st, msg = _create_error(TINY.replace(**change))
    assert st == status, msg
    assert needle in msg, msg


def test_create_rejects_token_counts_beyond_the_32_bit_k_offsets_of_bf16_attention():
    # rows of 2 * hidden bf16 values, addressed with 32-bit byte offsets inside a segment
    st, msg = _create_error(TINY, max_tokens=(1 << 30) // 64)
    assert st == B.EPD_ERR_UNSUPPORTED and "max_tokens * hidden" in msg, msg
    assert B.epd_encode_workspace_bytes(B.make_cfg(TINY, (1 << 30) // 64 - 1, 4, 4)) > 0


def test_create_rejects_segment_counts_beyond_the_32_bit_offsets_of_the_transposed_v_rows():
    # a head's V^T rows are head_dim rows of (max_tokens + 128 * max_segments) bf16 columns,
    # addressed with 32-bit byte offsets: many segments alone can push that past 2^32
    wide = TINY.replace(hidden=128, num_heads=1, head_dim=128, rope_pairs=(0, 32, 32))
    c = B.make_cfg(wide, 1 << 16, 140000, 4)
    assert B.epd_encode_workspace_bytes(c) == 0
    c = B.make_cfg(wide, 1 << 16, 100000, 4)
    assert B.epd_encode_workspace_bytes(c) > 0
    h = C.c_void_p()
    c = B.make_cfg(wide, 1 << 16, 140000, 4)
    assert B.lib.epd_encode_create(C.byref(c), C.byref(h)) == B.EPD_ERR_UNSUPPORTED
    assert "max_segments" in B.epd_encode_last_error(None)


def test_built_library_carries_the_hash_of_its_sources():
    """The binary the tests load is the one built from the sources as they stand: build() stores a
    hash of csrc/, the public header and the flags next to the library, and library_path() builds
    again when that stamp differs from the tree."""
    from paper_2601_11590_amd import build as bld
    assert os.path.exists(bld.LIB) and bld.built_hash() == bld.source_hash()
    assert bld.source_hash(("-DX",)) != bld.source_hash()


def test_create_rejects_bad_pointers_enums_and_workspace():
    st, msg = _create_error(TINY, lambda c: setattr(c, "struct_size", 12))
    assert st == B.EPD_ERR_INVALID_ARG and "struct_size" in msg
    st, msg = _create_error(TINY, lambda c: setattr(c, "dtype", 7))
    assert st == B.EPD_ERR_INVALID_ARG and "dtype" in msg
    st, msg = _create_error(TINY, lambda c: setattr(c, "norm", 5))
    assert st == B.EPD_ERR_INVALID_ARG and "norm" in msg
    st, msg = _create_error(TINY, lambda c: setattr(c, "rope", 1))
    assert st == B.EPD_ERR_INVALID_ARG and "rope" in msg
    st, msg = _create_error(TINY, with_buffers=False)
    assert st == B.EPD_ERR_INVALID_ARG and "weights" in msg
    st, msg = _create_error(TINY, lambda c: setattr(c, "workspace", 0x100010))
    assert st == B.EPD_ERR_WORKSPACE and "aligned" in msg
    st, msg = _create_error(TINY, lambda c: setattr(c, "workspace_bytes", 1024))
    assert st == B.EPD_ERR_WORKSPACE and "workspace_bytes" in msg
    assert B.lib.epd_encode_create(None, None) == B.EPD_ERR_INVALID_ARG
    # NULL handles are rejected by every entry point
    assert B.lib.epd_encode(None, None, None, 0, None, 0, None, None) == B.EPD_ERR_INVALID_ARG
    assert B.lib.epd_encode_destroy(None) == B.EPD_ERR_INVALID_ARG
    assert B.lib.epd_encode_set_timing(None, 0) == B.EPD_ERR_INVALID_ARG
    assert B.lib.epd_encode_set_tuning(None, -1, 0) == B.EPD_ERR_INVALID_ARG
    assert B.lib.epd_encode_set_compute_units(None, 224) == B.EPD_ERR_INVALID_ARG
    assert B.epd_encode_workspace_bytes(B.make_cfg(TINY.replace(head_dim=60), 64, 1, 1)) == 0


def test_product_path_never_touches_the_oracle():
    """The package must not import, read or execute anything under oracle/."""
    pkg = os.path.join(ROOT, "paper_2601_11590_amd")
    for base, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(base, f)).read()
                assert "oracle" not in text.replace("CPU oracle", "").replace("the oracle's callers", ""), f
    code = "import sys; import paper_2601_11590_amd.binding; assert not any(m.startswith('oracle') for m in sys.modules)"
    subprocess.run([sys.executable, "-c", code], check=True, cwd=ROOT)


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message (this build runs on exactly one GPU); it must
    do so before touching the GPU, so the check runs anywhere."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_workspace_pads_mlp_width_and_keeps_a_read_tail():
    """bf16 workspaces grow with a padded MLP width (4304 -> 4352 columns of hidden activations and
    fc2 weights) and hold a tail behind the last buffer; fp32 ones do neither."""
    base = dict(name="w", num_layers=1, hidden=128, num_heads=2, head_dim=64, patch=4, temporal_patch=1,
                norm="layernorm", rope="2d", rope_pairs=(0, 16, 16), out_dim=64, seed=1)
    sizes = {}
    for dtype in ("bf16", "f32"):
        for mlp in (128, 136):
            cfg = W.EncoderConfig(dtype=dtype, mlp_dim=mlp, **base)
            sizes[dtype, mlp] = B.epd_encode_workspace_bytes(B.make_cfg(cfg, 256, 4, 4))
            assert sizes[dtype, mlp] > 0
    es = 2
    # 136 pads to 192 columns: (192 - 128) more columns of Hd (256 tokens) and of fc2_w (128 rows),
    # fc1 rows grow by 8 without padding; everything is rounded up to 256-byte blocks
    grow_bf16 = sizes["bf16", 136] - sizes["bf16", 128]
    assert grow_bf16 >= (256 + 128) * 64 * es
    grow_f32 = sizes["f32", 136] - sizes["f32", 128]
    assert 0 < grow_f32 <= (256 + 128 + 128 + 1) * 8 * 4 + 4 * 256


def test_gemm_launch_planner_on_the_benchmark_shapes():
    """Host logic of the bf16 GEMM launcher, read through its probe for a 256-unit chip: one
    launch of a large tile where its rounds come out whole, the 320 x 256 tile where it saves a
    round or K is short, 128 x 128 tiles on narrow outputs and for short-K GEMMs with a heavy
    epilogue, and a large-tile body plus a small-tile tail where the last round of large tiles
    would be partial."""
    from paper_2601_11590_amd import binding as B
    plan = lambda *a: B.epd_probe_gemm_plan(*a, compute_units=256)
    G, R, Q = B.EPI_GELU, B.EPI_RESIDUAL, B.EPI_QKV
    # C5 (32 768 tokens, hidden 3200, MLP 12 800): fc1 = 6400 256 x 256 tiles = 25 whole rounds (or 20
    # rounds of 320 x 256 + a 128-row tail), QKV = 19 whole rounds
    assert plan(32768, 12800, 3200, G) in ((256, 256, 0), (320, 256, 32640))     # priced within 2 % of each other
    assert plan(32768, 9600, 3200, Q, 6400) == (256, 256, 0)
    # ... proj / fc2: 1664 tiles = 6.5 rounds -> 6 rounds over 30 208 rows + small tiles
    assert plan(32768, 3200, 3200, R) == (256, 256, 30208)
    assert plan(32768, 3200, 12800, R) == (256, 256, 30208)
    # C2 (6272 tokens, hidden 1024): QKV is ONE round of 240 320 x 256 tiles; N = 1024 -> 128 x 128;
    # fc1 = one round of 320 x 256 tiles over 5120 rows + small tiles instead of two rounds of 256 x 256
    assert plan(6272, 3072, 1024, Q, 2048) == (320, 256, 0)
    assert plan(6272, 1024, 1024, R) == (128, 128, 0)
    assert plan(6272, 4096, 1024, G) == (320, 256, 5120)
    # C3 (73 896 tokens, hidden 1024): the residual epilogue against K = 1024 goes to the small tile,
    # against K = 4096 to four rounds of 320 x 256 instead of five of 256 x 256
    assert plan(73896, 1024, 1024, R) == (128, 128, 0)
    assert plan(73896, 1024, 4096, R) == (320, 256, 0)
    # Q | K columns that do not end on a 256-column boundary: the 256 x 128 tile, never cut
    assert plan(13540, 960, 320, Q, 640) == (256, 128, 0)
    # a QKV projection that is cut (9124 x 2304 at K = 768)
    assert plan(9124, 2304, 768, Q, 1536) == (256, 256, 7168)
    # a chip with fewer units changes the rounds, hence the plan
    assert plan(32768, 3200, 3200, R) != B.epd_probe_gemm_plan(32768, 3200, 3200, R, compute_units=208)
    for bad in [(0, 128, 64), (128, 0, 64), (128, 128, 0), (128, 128, 64, 4), (128, 128, 64, -1), (128, 128, 64, Q, 0), (128, 128, 64, Q, 256)]:
        with pytest.raises(B.EpdError):
            B.epd_probe_gemm_plan(*bad, compute_units=256)
