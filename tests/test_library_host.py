"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its
host logic (sizes, selection counts, argument validation) works without a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import hero_oracle as O
from paper_2508_17588_amd import binding as B
from workloads import CONFIGS, RATIO_SWEEP, get_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2508_17588_amd.build import build
        build(verbose=False)
    return B.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hero.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hero_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    names = declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), f"{n} declared in hero.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_config_struct_layout_matches_header(lib):
    # 16 int32/float fields, a uint64 seed, then select_mode, block_flags, cache_flags, debug_flags: 88 bytes
    assert ctypes.sizeof(B.hero_config) == 88
    assert B.hero_config.cache_flags.offset == 80 and B.hero_config.debug_flags.offset == 84
    assert B.hero_config.seed.offset == 64
    assert B.hero_config.select_mode.offset == 72
    assert ctypes.sizeof(B.hero_layer_weights) == 17 * ctypes.sizeof(ctypes.c_void_p)


@pytest.mark.parametrize("name", sorted(CONFIGS))
def test_num_selected_matches_oracle_count(lib, name):
    cfg = get_config(name)
    want = sum(O.tokens_per_patch(cfg.ratio, hh * ww) for (_, _, _, hh, ww) in
               O.patch_list(cfg.frames, cfg.height, cfg.width, cfg.patch_h, cfg.patch_w))
    assert B.hero_num_selected(B.make_config(cfg)) == want


def test_num_selected_ratio_sweep_and_odd_grids(lib):
    for over in list(RATIO_SWEEP.values()) + [dict(height=7, width=9, patch_h=2, patch_w=3, ratio=0.34),
                                               dict(height=5, width=5, patch_h=3, patch_w=2, ratio=0.5),
                                               dict(ratio=0.0), dict(ratio=1.0), dict(patch_h=64, patch_w=64)]:
        cfg = get_config("cvx5b_block", **over)
        want = sum(O.tokens_per_patch(cfg.ratio, hh * ww) for (_, _, _, hh, ww) in
                   O.patch_list(cfg.frames, cfg.height, cfg.width, cfg.patch_h, cfg.patch_w))
        assert B.hero_num_selected(B.make_config(cfg)) == want


def test_cache_bytes(lib):
    cfg = get_config("cvx5b_42l")
    cb, wb = B.hero_cache_bytes(B.make_config(cfg))
    n, d = cfg.n_tokens, cfg.hidden
    n_pad = (n + 63) // 64 * 64
    s = n * d * 2
    want = cfg.n_shallow * (2 * s + d * n_pad * 2) + (cfg.n_layers - cfg.n_shallow) * 2 * s
    want += 2 * n * d * 4          # two fp32 sums over the deep layers (one per full-step generation)
    assert want <= cb <= want + 256 * 200 + cfg.n_video * 4
    assert wb >= 3 * s + n * cfg.ffn_dim * 2
    assert cb + wb < 40e9          # far below one GPU's 288 GB
    # rotary positions add a (cos, sin) table: one float pair per video token and channel pair
    cb_rope, _ = B.hero_cache_bytes(B.make_config(cfg.with_(block_flags=4)))
    table = cfg.n_video * (cfg.head_dim // 2) * 8
    assert table <= cb_rope - cb <= table + 256
    # adaLN and q/k normalisation need no cache memory of their own
    assert B.hero_cache_bytes(B.make_config(cfg.with_(block_flags=3)))[0] == cb


def test_invalid_configs_are_rejected(lib):
    def rc_of(**over):
        c = B.make_config(get_config("tiny", **over))
        n = ctypes.c_int32(0)
        return lib.hero_num_selected(ctypes.byref(c), ctypes.byref(n))
    assert rc_of() == B.HERO_OK
    assert rc_of(n_layers=0) == B.HERO_ERR_INVALID_ARG
    assert rc_of(n_shallow=3) == B.HERO_ERR_INVALID_ARG
    assert rc_of(interval=0) == B.HERO_ERR_INVALID_ARG
    assert rc_of(patch_h=0) == B.HERO_ERR_INVALID_ARG
    assert rc_of(ratio=-0.5) == B.HERO_ERR_INVALID_ARG
    assert rc_of(select_mode=2) == B.HERO_ERR_INVALID_ARG
    assert rc_of(select_mode=1) == B.HERO_OK
    assert rc_of(block_flags=7) == B.HERO_OK
    assert rc_of(block_flags=8) == B.HERO_ERR_INVALID_ARG
    assert rc_of(cache_flags=3) == B.HERO_OK and rc_of(cache_flags=4) == B.HERO_ERR_INVALID_ARG
    assert rc_of(debug_flags=1) == B.HERO_OK and rc_of(debug_flags=2) == B.HERO_ERR_INVALID_ARG
    assert rc_of(select_mode=1, height=300, width=300, patch_h=256, patch_w=257) == B.HERO_ERR_SHAPE
    assert rc_of(head_dim=48, n_heads=4, hidden=192) == B.HERO_ERR_SHAPE
    assert rc_of(hidden=96, n_heads=3) == B.HERO_ERR_SHAPE           # not a multiple of 64
    assert rc_of(hidden=128, n_heads=3) == B.HERO_ERR_SHAPE          # hidden != heads * head_dim
    assert rc_of(ffn_dim=100) == B.HERO_ERR_SHAPE
    assert b"multiple" in lib.hero_last_error()
    # 32-bit operand offsets: (tokens + 512) * max(hidden, ffn_dim) * 2 < 2^32
    assert rc_of(frames=1, height=2048, width=2500) == B.HERO_ERR_SHAPE      # 5.1 M tokens x ffn 512
    assert b"32-bit" in lib.hero_last_error()

    def rc_5b(frames):
        c = B.make_config(get_config("cvx5b_block", frames=frames))
        n = ctypes.c_int32(0)
        return lib.hero_num_selected(ctypes.byref(c), ctypes.byref(n))
    assert rc_5b(128) == B.HERO_OK                # 173 026 tokens x ffn 12288: 4.265e9 bytes
    assert rc_5b(134) == B.HERO_ERR_SHAPE         # 181 126 tokens: beyond
    assert lib.hero_num_selected(None, None) == B.HERO_ERR_INVALID_ARG


def test_null_and_small_buffers_are_rejected_before_any_gpu_work(lib):
    c = B.make_config(get_config("tiny"))
    h = ctypes.c_void_p(0)
    rc = lib.hero_cache_create(ctypes.byref(c), None, 0, None, 0, None, ctypes.byref(h))
    assert rc == B.HERO_ERR_INVALID_ARG
    rc = lib.hero_cache_create(ctypes.byref(c), ctypes.c_void_p(256), 16, ctypes.c_void_p(512), 16, None, ctypes.byref(h))
    assert rc == B.HERO_ERR_BUFFER_TOO_SMALL and b"needed" in lib.hero_last_error()
    rc = lib.hero_cache_create(ctypes.byref(c), ctypes.c_void_p(260), 1 << 40, ctypes.c_void_p(512), 1 << 40, None, ctypes.byref(h))
    assert rc == B.HERO_ERR_INVALID_ARG      # misaligned
    for fn, args in ((lib.hero_cache_destroy, (None,)), (lib.hero_cache_reset, (None, None)),
                     (lib.hero_step, (None, None, 0, None)), (lib.hero_full_layer, (None, 0, None, None)),
                     (lib.hero_refresh_layer, (None, 0, None, None, 0, None)),
                     (lib.hero_extrapolate_layer, (None, 0, None, 1, None))):
        assert fn(*args) == B.HERO_ERR_INVALID_ARG
    assert lib.hero_linear(None, None, None, None, 1, 64, 64, 0, None) == B.HERO_ERR_INVALID_ARG
    p = ctypes.c_void_p(256)
    assert lib.hero_linear(p, p, p, p, 1, 60, 64, 0, None) == B.HERO_ERR_SHAPE
    assert lib.hero_linear_scratch(p, p, p, p, 1, 64, 64, 0, ctypes.c_void_p(260), 1 << 20, None) == B.HERO_ERR_INVALID_ARG
    # the no-allocation GEMM refuses a k-split that its own 32 MiB array cannot hold, before any launch
    assert lib.hero_linear_static(p, p, p, p, 17776, 3072, 12288, 0, None) == B.HERO_ERR_BUFFER_TOO_SMALL
    assert b"hero_linear_scratch" in lib.hero_last_error()
    assert lib.hero_linear_static(p, p, p, p, 1, 60, 64, 0, None) == B.HERO_ERR_SHAPE
    # misaligned operands
    q = ctypes.c_void_p(264)
    assert lib.hero_linear(q, p, p, p, 1, 64, 64, 0, None) == B.HERO_ERR_INVALID_ARG
    assert lib.hero_attention(p, q, p, 128, p, 1, 100, 1, 64, None) == B.HERO_ERR_INVALID_ARG
    assert lib.hero_axpy_features(p, 1, q, None, 0.0, 16, None) == B.HERO_ERR_INVALID_ARG
    assert lib.hero_gather_ln(p, 1, None, None, 1, 64, p, q, 1e-5, p, None) == B.HERO_ERR_INVALID_ARG
    assert lib.hero_attention(p, p, p, 100, p, 1, 100, 1, 64, None) == B.HERO_ERR_SHAPE
    assert lib.hero_attention(p, p, p, 128, p, 1, 100, 1, 48, None) == B.HERO_ERR_SHAPE
    # operand sizes beyond the kernels' 32-bit offsets
    assert lib.hero_linear(p, p, p, p, 699_051, 256, 3072, 0, None) == B.HERO_ERR_SHAPE
    assert b"2^32" in lib.hero_last_error()
    assert lib.hero_linear(p, p, p, p, 64, 699_051 // 64 * 64 + 64, 3072, 0, None) == B.HERO_ERR_SHAPE
    assert lib.hero_attention(p, p, p, 699_136, p, 1, 699_100, 48, 64, None) == B.HERO_ERR_SHAPE
    assert b"2^32" in lib.hero_last_error()
    assert lib.hero_axpy_features(p, 1, p, None, 0.0, 12, None) == B.HERO_ERR_SHAPE
    assert lib.hero_gather_ln(p, 7, None, None, 1, 64, p, p, 1e-5, p, None) == B.HERO_ERR_INVALID_ARG


def test_stability_scores_host_function_matches_oracle(lib):
    v = [4.0, 1.0, 2.5, 1.0, 3.25]
    np.testing.assert_allclose(B.hero_stability_scores(v), O.stability_scores(v), rtol=0, atol=1e-15)
    np.testing.assert_allclose(B.hero_stability_scores([2.0, 2.0]), [1.0, 1.0])
    out = (ctypes.c_double * 2)()
    bad = (ctypes.c_double * 2)(1.0, -1.0)
    assert lib.hero_stability_scores(bad, 2, out) == B.HERO_ERR_INVALID_ARG
    assert lib.hero_stability_scores(None, 2, out) == B.HERO_ERR_INVALID_ARG
    p = ctypes.c_void_p(256)
    assert lib.hero_second_diff_stats(p, p, p, 12, p, 1 << 20, p, 0, None) == B.HERO_ERR_SHAPE
    assert lib.hero_second_diff_stats(p, p, p, 16, p, 64, p, 0, None) == B.HERO_ERR_BUFFER_TOO_SMALL
    assert lib.hero_second_diff_stats(p, p, None, 16, p, 1 << 20, p, 0, None) == B.HERO_ERR_INVALID_ARG


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_17588_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no CPU or PyTorch fallback", ""), f
