"""ctypes binding of libhero.so: argument marshalling only.

Every function mirrors an entry point declared in include/hero.h under the same
name.  Tensors are torch CUDA(ROCm) tensors used purely as device buffers; the
stream passed down is torch's current stream.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char_p, c_float, c_int32, c_int64, c_size_t,
                    c_uint64, c_void_p)
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhero.so")

HERO_OK = 0
HERO_ERR_INVALID_ARG = 1
HERO_ERR_SHAPE = 2
HERO_ERR_STATE = 3
HERO_ERR_BUFFER_TOO_SMALL = 4
HERO_ERR_HIP = 5
DTYPE_BF16 = 0
DTYPE_FP32 = 1

VIEW_S_CUR, VIEW_S_PREV, VIEW_K, VIEW_VT, VIEW_AGES, VIEW_IDX, VIEW_FALLBACKS = range(7)

PROF_KINDS = ("select", "ln", "gemm_qkv", "attention", "gemm_o", "gemm_ff1", "gemm_ff2", "resid", "extrap", "deepsum", "qk_post")

WEIGHT_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                 "ln2_g", "ln2_b", "w_ff1", "b_ff1", "w_ff2", "b_ff2")
EXTRA_WEIGHT_FIELDS = ("q_norm_g", "q_norm_b", "k_norm_g", "k_norm_b", "mod")
BLOCK_ADALN, BLOCK_QKNORM, BLOCK_ROPE = 1, 2, 4
CACHE_KV_ALL_LAYERS, CACHE_PREV_ALL_LAYERS = 1, 2
DEBUG_CHECK_IDX = 1

EXPORTS = (
    "hero_last_error", "hero_num_selected", "hero_cache_bytes", "hero_cache_create",
    "hero_cache_destroy", "hero_cache_reset", "hero_set_layer_weights", "hero_full_layer",
    "hero_select", "hero_reset_ages", "hero_refresh_layer", "hero_extrapolate_layer", "hero_step",
    "hero_cache_view", "hero_cache_state", "hero_profile_begin", "hero_profile_begin_kinds", "hero_profile_end", "hero_gather_ln", "hero_linear", "hero_linear_scratch", "hero_linear_static",
    "hero_attention", "hero_attention_scratch", "hero_attention_counted",
    "hero_axpy_features", "hero_second_diff_stats", "hero_stability_scores",
)


class HeroError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"hero error {code}: {msg}")
        self.code = code


class hero_config(Structure):
    _fields_ = [("n_layers", c_int32), ("n_shallow", c_int32), ("interval", c_int32),
                ("hidden", c_int32), ("n_heads", c_int32), ("head_dim", c_int32), ("ffn_dim", c_int32),
                ("frames", c_int32), ("height", c_int32), ("width", c_int32), ("n_text", c_int32),
                ("patch_h", c_int32), ("patch_w", c_int32), ("ratio", c_float),
                ("resid_dtype", c_int32), ("ln_eps", c_float), ("seed", c_uint64),
                ("select_mode", c_int32), ("block_flags", c_int32),
                ("cache_flags", c_int32), ("debug_flags", c_int32)]


class hero_layer_weights(Structure):
    _fields_ = [(n, c_void_p) for n in WEIGHT_FIELDS + EXTRA_WEIGHT_FIELDS]


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads libhero.so (raises if it has not been built)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise FileNotFoundError(f"{p} not found: build it with `python -m paper_2508_17588_amd.build`")
    lib = ctypes.CDLL(p)
    lib.hero_last_error.restype = c_char_p
    lib.hero_last_error.argtypes = []
    I, P = c_int32, c_void_p
    sig = {
        "hero_num_selected": [POINTER(hero_config), POINTER(c_int32)],
        "hero_cache_bytes": [POINTER(hero_config), POINTER(c_size_t), POINTER(c_size_t)],
        "hero_cache_create": [POINTER(hero_config), P, c_size_t, P, c_size_t, P, POINTER(c_void_p)],
        "hero_cache_destroy": [P],
        "hero_cache_reset": [P, P],
        "hero_set_layer_weights": [P, I, POINTER(hero_layer_weights)],
        "hero_full_layer": [P, I, P, P],
        "hero_select": [P, I, P, POINTER(c_int32), P],
        "hero_reset_ages": [P, P],
        "hero_refresh_layer": [P, I, P, P, I, P],
        "hero_extrapolate_layer": [P, I, P, I, P],
        "hero_step": [P, P, I, P],
        "hero_cache_view": [P, I, I, POINTER(c_void_p), POINTER(c_int64)],
        "hero_cache_state": [P, POINTER(c_int32), POINTER(c_int32)],
        "hero_profile_begin": [P],
        "hero_profile_begin_kinds": [P, ctypes.c_uint32],
        "hero_profile_end": [P, P, POINTER(ctypes.c_double), POINTER(c_int64), POINTER(ctypes.c_double)],
        "hero_gather_ln": [P, I, P, P, I, I, P, P, c_float, P, P],
        "hero_linear": [P, P, P, P, I, I, I, I, P],
        "hero_linear_scratch": [P, P, P, P, I, I, I, I, P, ctypes.c_size_t, P],
        "hero_linear_static": [P, P, P, P, I, I, I, I, P],
        "hero_attention": [P, P, P, c_int64, P, I, I, I, I, P],
        "hero_attention_scratch": [P, P, P, c_int64, P, I, I, I, I, P, ctypes.c_size_t, P],
        "hero_attention_counted": [P, P, P, c_int64, P, I, I, I, I, P, ctypes.c_size_t, P, P],
        "hero_axpy_features": [P, I, P, P, c_float, c_int64, P],
        "hero_second_diff_stats": [P, P, P, c_int64, P, ctypes.c_size_t, P, I, P],
        "hero_stability_scores": [POINTER(ctypes.c_double), I, POINTER(ctypes.c_double)],
    }
    for name, argtypes in sig.items():
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = argtypes
    if path is None:
        _lib = lib
    return lib


def _check(rc: int):
    if rc != HERO_OK:
        raise HeroError(rc, load_library().hero_last_error().decode())


def make_config(cfg, resid_fp32: Optional[bool] = None) -> hero_config:
    """hero_config from a workloads.HeroConfig-like object."""
    rf = cfg.resid_fp32 if resid_fp32 is None else resid_fp32
    return hero_config(cfg.n_layers, cfg.n_shallow, cfg.interval, cfg.hidden, cfg.n_heads, cfg.head_dim,
                       cfg.ffn_dim, cfg.frames, cfg.height, cfg.width, cfg.n_text, cfg.patch_h, cfg.patch_w,
                       cfg.ratio, DTYPE_FP32 if rf else DTYPE_BF16, cfg.ln_eps, cfg.seed,
                       getattr(cfg, "select_mode", 0), getattr(cfg, "block_flags", 0),
                       getattr(cfg, "cache_flags", 0), getattr(cfg, "debug_flags", 0))


def _stream() -> c_void_p:
    import torch
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t) -> c_void_p:
    return c_void_p(0) if t is None else c_void_p(t.data_ptr())


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return DTYPE_FP32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError(f"unsupported activation dtype {t.dtype}")


def _need(t, dtype, name):
    if t.dtype != dtype or not t.is_cuda or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous {dtype} device tensor")


def hero_num_selected(cfg: hero_config) -> int:
    n = c_int32(0)
    _check(load_library().hero_num_selected(byref(cfg), byref(n)))
    return n.value


def hero_cache_bytes(cfg: hero_config):
    a, b = c_size_t(0), c_size_t(0)
    _check(load_library().hero_cache_bytes(byref(cfg), byref(a), byref(b)))
    return a.value, b.value


class HeroCache:
    """Owns the two device buffers (torch uint8 tensors) and the library handle."""

    def __init__(self, cfg: hero_config, device="cuda:0"):
        import torch
        self.lib = load_library()
        self.cfg = cfg
        cb, wb = hero_cache_bytes(cfg)
        self.cache_buf = torch.empty(cb, dtype=torch.uint8, device=device)
        self.ws_buf = torch.empty(wb, dtype=torch.uint8, device=device)
        self.handle = c_void_p(0)
        self._weights = []   # keeps the parameter tensors alive
        _check(self.lib.hero_cache_create(byref(cfg), _ptr(self.cache_buf), cb, _ptr(self.ws_buf), wb,
                                          _stream(), byref(self.handle)))
        self.n_video = cfg.frames * cfg.height * cfg.width
        self.n_tokens = self.n_video + cfg.n_text
        self.x_dtype = torch.float32 if cfg.resid_dtype == DTYPE_FP32 else torch.bfloat16

    def close(self):
        if self.handle:
            self.lib.hero_cache_destroy(self.handle)
            self.handle = c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _x(self, x):
        _need(x, self.x_dtype, "x")
        if x.numel() != self.n_tokens * self.cfg.hidden:
            raise ValueError("x must be [n_tokens, hidden]")
        return _ptr(x)

    def hero_cache_reset(self):
        _check(self.lib.hero_cache_reset(self.handle, _stream()))

    def hero_set_layer_weights(self, layer: int, w: Dict[str, "object"]):
        import torch
        st = hero_layer_weights()
        for n in WEIGHT_FIELDS:
            _need(w[n], torch.bfloat16, n)
            setattr(st, n, w[n].data_ptr())
        for n in EXTRA_WEIGHT_FIELDS:          # only needed with the matching block flag
            if w.get(n) is not None:
                _need(w[n], torch.bfloat16, n)
                setattr(st, n, w[n].data_ptr())
        self._weights.append(w)
        _check(self.lib.hero_set_layer_weights(self.handle, layer, byref(st)))

    def hero_full_layer(self, layer: int, x):
        _check(self.lib.hero_full_layer(self.handle, layer, self._x(x), _stream()))

    def hero_select(self, step: int, idx) -> int:
        import torch
        _need(idx, torch.int32, "idx")
        if idx.numel() < hero_num_selected(self.cfg):
            raise ValueError("idx buffer too small")
        n = c_int32(0)
        _check(self.lib.hero_select(self.handle, step, _ptr(idx), byref(n), _stream()))
        return n.value

    def hero_reset_ages(self):
        _check(self.lib.hero_reset_ages(self.handle, _stream()))

    def hero_refresh_layer(self, layer: int, x, idx, n_sel: int):
        import torch
        if idx is not None:
            _need(idx, torch.int32, "idx")
            if idx.numel() < n_sel:
                raise ValueError("idx shorter than n_sel")
        _check(self.lib.hero_refresh_layer(self.handle, layer, self._x(x), _ptr(idx), n_sel, _stream()))

    def hero_extrapolate_layer(self, layer: int, x, k: int):
        _check(self.lib.hero_extrapolate_layer(self.handle, layer, self._x(x), k, _stream()))

    def hero_step(self, x, step: int):
        _check(self.lib.hero_step(self.handle, self._x(x), step, _stream()))

    def hero_cache_state(self):
        a, b = c_int32(0), c_int32(0)
        _check(self.lib.hero_cache_state(self.handle, byref(a), byref(b)))
        return a.value, b.value

    def hero_profile_begin(self):
        _check(self.lib.hero_profile_begin(self.handle))

    def hero_profile_begin_kinds(self, kinds):
        """Bracket only the named kinds (entries of PROF_KINDS)."""
        mask = 0
        for k in kinds:
            mask |= 1 << PROF_KINDS.index(k)
        _check(self.lib.hero_profile_begin_kinds(self.handle, mask))

    def hero_profile_end(self):
        """-> {slot_name: (ms, launches, work)}; slot names end in '/full' or '/cached'."""
        n = 2 * len(PROF_KINDS)
        ms, cnt, work = (ctypes.c_double * n)(), (c_int64 * n)(), (ctypes.c_double * n)()
        _check(self.lib.hero_profile_end(self.handle, _stream(), ms, cnt, work))
        out = {}
        for i in range(n):
            if cnt[i]:
                name = PROF_KINDS[i % len(PROF_KINDS)] + ("/full" if i < len(PROF_KINDS) else "/cached")
                out[name] = (ms[i], cnt[i], work[i])
        return out

    def hero_cache_view(self, layer: int, what: int):
        """Returns a torch tensor aliasing the cache slab (no copy)."""
        import torch
        p, ld = c_void_p(0), c_int64(0)
        _check(self.lib.hero_cache_view(self.handle, layer, what, byref(p), byref(ld)))
        cfg = self.cfg
        if what in (VIEW_AGES, VIEW_IDX, VIEW_FALLBACKS):
            base, dtype, shape, esz = self.cache_buf if what == VIEW_AGES else self.ws_buf, torch.int32, (ld.value,), 4
        elif what == VIEW_VT:
            base, dtype, shape, esz = self.cache_buf, torch.bfloat16, (cfg.hidden, ld.value), 2
        else:
            base, dtype, shape, esz = self.cache_buf, torch.bfloat16, (self.n_tokens, cfg.hidden), 2
        off = p.value - base.data_ptr()
        n = 1
        for s in shape:
            n *= s
        return base[off:off + n * esz].view(dtype).view(*shape)


# ---- building blocks ----------------------------------------------------------------

def hero_gather_ln(x, add, rows, n_rows: int, gain, bias, eps: float, out):
    import torch
    hidden = x.shape[-1]
    _need(out, torch.bfloat16, "out")
    if out.numel() < n_rows * hidden:
        raise ValueError("out too small")
    if rows is not None:
        _need(rows, torch.int32, "rows")
    _check(load_library().hero_gather_ln(_ptr(x), _dtype_code(x), _ptr(add), _ptr(rows), n_rows, hidden,
                                         _ptr(gain), _ptr(bias), eps, _ptr(out), _stream()))


def hero_linear(a, w, bias, c, act: int = 0):
    import torch
    for t, n in ((a, "a"), (w, "w"), (bias, "bias"), (c, "c")):
        _need(t, torch.bfloat16, n)
    m, k = a.shape
    n = w.shape[0]
    if w.shape[1] != k or bias.numel() != n or c.numel() < m * n:
        raise ValueError("shape mismatch")
    _check(load_library().hero_linear(_ptr(a), _ptr(w), _ptr(bias), _ptr(c), m, n, k, act, _stream()))


def hero_linear_scratch(a, w, bias, c, scratch, act: int = 0):
    """hero_linear with a caller-owned device scratch tensor (any dtype, contiguous)."""
    import torch
    for t, n in ((a, "a"), (w, "w"), (bias, "bias"), (c, "c")):
        _need(t, torch.bfloat16, n)
    m, k = a.shape
    n = w.shape[0]
    if w.shape[1] != k or bias.numel() != n or c.numel() < m * n:
        raise ValueError("shape mismatch")
    if not scratch.is_cuda or not scratch.is_contiguous():
        raise ValueError("scratch must be a contiguous device tensor")
    _check(load_library().hero_linear_scratch(_ptr(a), _ptr(w), _ptr(bias), _ptr(c), m, n, k, act, _ptr(scratch),
                                              scratch.numel() * scratch.element_size(), _stream()))


def hero_linear_static(a, w, bias, c, act: int = 0):
    """hero_linear_scratch with the library's own 32 MiB scratch: the call allocates nothing."""
    import torch
    for t, n in ((a, "a"), (w, "w"), (bias, "bias"), (c, "c")):
        _need(t, torch.bfloat16, n)
    m, k = a.shape
    n = w.shape[0]
    if w.shape[1] != k or bias.numel() != n or c.numel() < m * n:
        raise ValueError("shape mismatch")
    _check(load_library().hero_linear_static(_ptr(a), _ptr(w), _ptr(bias), _ptr(c), m, n, k, act, _stream()))


def hero_attention(q, k, vt, o, n_keys: int, n_heads: int, head_dim: int, scratch=None, fallbacks=None):
    """scratch: optional contiguous device tensor; with it the call goes through hero_attention_scratch.
    fallbacks: optional int32 device tensor of one element; the call then goes through
    hero_attention_counted and adds the number of workgroups that took the running-maximum path."""
    import torch
    for t, n in ((q, "q"), (k, "k"), (vt, "vt"), (o, "o")):
        _need(t, torch.bfloat16, n)
    r = q.shape[0]
    d = n_heads * head_dim
    if q.shape[1] != d or k.shape[1] != d or k.shape[0] < n_keys or vt.shape[0] != d or o.numel() < r * d:
        raise ValueError("shape mismatch")
    if fallbacks is not None:
        _need(fallbacks, torch.int32, "fallbacks")
        _check(load_library().hero_attention_counted(_ptr(q), _ptr(k), _ptr(vt), vt.shape[1], _ptr(o), r, n_keys,
                                                     n_heads, head_dim, _ptr(scratch),
                                                     0 if scratch is None else scratch.numel() * scratch.element_size(),
                                                     _ptr(fallbacks), _stream()))
        return
    if scratch is not None:
        _check(load_library().hero_attention_scratch(_ptr(q), _ptr(k), _ptr(vt), vt.shape[1], _ptr(o), r, n_keys,
                                                     n_heads, head_dim, _ptr(scratch),
                                                     scratch.numel() * scratch.element_size(), _stream()))
        return
    _check(load_library().hero_attention(_ptr(q), _ptr(k), _ptr(vt), vt.shape[1], _ptr(o), r, n_keys,
                                         n_heads, head_dim, _stream()))


def hero_axpy_features(x, s_cur, s_prev, alpha: float):
    import torch
    _need(s_cur, torch.bfloat16, "s_cur")
    if s_prev is not None:
        _need(s_prev, torch.bfloat16, "s_prev")
        if s_prev.numel() != x.numel():
            raise ValueError("shape mismatch")
    if s_cur.numel() != x.numel() or not x.is_contiguous():
        raise ValueError("shape mismatch")
    _check(load_library().hero_axpy_features(_ptr(x), _dtype_code(x), _ptr(s_cur), _ptr(s_prev), alpha,
                                             x.numel(), _stream()))


def hero_second_diff_stats(f_prev, f_cur, f_next, scratch, stats, accumulate: bool = False):
    """stats (float64[2] device tensor) (+)= [sum D, sum D^2] with D = f_next - 2 f_cur + f_prev."""
    import torch
    for t, n in ((f_prev, "f_prev"), (f_cur, "f_cur"), (f_next, "f_next")):
        _need(t, torch.bfloat16, n)
    if f_prev.numel() != f_cur.numel() or f_next.numel() != f_cur.numel():
        raise ValueError("shape mismatch")
    if stats.dtype != torch.float64 or stats.numel() < 2 or not stats.is_cuda or not scratch.is_cuda:
        raise ValueError("stats must be a float64 device tensor of 2 elements, scratch a device tensor")
    _check(load_library().hero_second_diff_stats(_ptr(f_prev), _ptr(f_cur), _ptr(f_next), f_cur.numel(), _ptr(scratch),
                                                 scratch.numel() * scratch.element_size(), _ptr(stats),
                                                 1 if accumulate else 0, _stream()))


def hero_stability_scores(variances):
    n = len(variances)
    v = (ctypes.c_double * n)(*[float(a) for a in variances])
    out = (ctypes.c_double * n)()
    _check(load_library().hero_stability_scores(v, n, out))
    return list(out)
