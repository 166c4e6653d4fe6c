"""Seeded synthetic workloads for the cached DiT denoising step (HERO).

This module is the one thing the CPU oracle and the HIP path share: it
describes workload shapes and draws seeded synthetic inputs.  It holds none of
the method's arithmetic (no LayerNorm, attention, selection, extrapolation) --
only shapes, random draws, bf16 value rounding of the drawn inputs, and the
harness-defined toy sampler update that stands between two denoising steps.

The token-grid shapes stand in for the paper's Aether / CogVideoX workloads
(a 480x720 CogVideoX latent gives a 30x45 token grid per latent frame, with
226 text tokens); no dataset item or trained weight is used anywhere.
"""
from __future__ import annotations

from dataclasses import dataclass, replace, asdict
from typing import Dict

import numpy as np

__all__ = [
    "HeroConfig", "CONFIGS", "get_config", "round_to_bf16", "bf16_bits",
    "from_bf16_bits", "make_layer_weights", "make_tokens", "perturb_tokens",
    "euler_update", "WEIGHT_NAMES", "make_block_extras", "MOD_ROWS", "BLOCK_ADALN", "BLOCK_QKNORM", "BLOCK_ROPE",
]


@dataclass(frozen=True)
class HeroConfig:
    """Shape + schedule description of one workload (paper Sec. 3, Alg. 1).

    n_layers L, n_shallow K (layers l < K refresh, l >= K extrapolate),
    interval M (a full step every M-th step), token grid frames x height x
    width (f, h', w') plus n_text text tokens placed first in the joint
    sequence, spatial patch patch_h x patch_w and sampling ratio R.
    """
    name: str
    n_layers: int
    n_shallow: int
    interval: int
    hidden: int
    n_heads: int
    head_dim: int
    ffn_dim: int
    frames: int
    height: int
    width: int
    n_text: int
    patch_h: int
    patch_w: int
    ratio: float
    n_steps: int = 1
    ln_eps: float = 1e-5
    seed: int = 1234          # selection seed
    resid_fp32: bool = True   # residual stream x kept in fp32 on the GPU
    select_mode: int = 0      # 0: age-priority selection, 1: age-weighted random sampling (Sec. 3.3)
    block_flags: int = 0      # bit 0: adaLN shift/scale/gate, bit 1: per-head q/k LayerNorm, bit 2: 3-D rotary positions
    cache_flags: int = 0      # bit 0: K/V kept on every layer, bit 1: previous generation kept on every layer
    debug_flags: int = 0      # bit 0: the refresh entry point verifies its index list on the device

    @property
    def n_video(self) -> int:
        return self.frames * self.height * self.width

    @property
    def n_tokens(self) -> int:
        return self.n_text + self.n_video

    def with_(self, **kw) -> "HeroConfig":
        return replace(self, **kw)

    def as_dict(self) -> dict:
        return asdict(self)


def _cfg(**kw) -> HeroConfig:
    return HeroConfig(**kw)


CONFIGS: Dict[str, HeroConfig] = {
    # config 1: tiny CPU-checkable DiT, 2 blocks (block 0 refresh, block 1 extrapolate)
    "tiny": _cfg(name="tiny", n_layers=2, n_shallow=1, interval=4, hidden=128,
                 n_heads=4, head_dim=32, ffn_dim=512, frames=4, height=8, width=8,
                 n_text=16, patch_h=2, patch_w=2, ratio=0.25, n_steps=10),
    # config 2: one CogVideoX-2B-shaped block
    "cvx2b_block": _cfg(name="cvx2b_block", n_layers=1, n_shallow=1, interval=2,
                        hidden=1920, n_heads=30, head_dim=64, ffn_dim=7680,
                        frames=13, height=30, width=45, n_text=226,
                        patch_h=2, patch_w=2, ratio=0.25, n_steps=2),
    # config 3: one CogVideoX-5B-shaped block (ratio swept via with_())
    "cvx5b_block": _cfg(name="cvx5b_block", n_layers=1, n_shallow=1, interval=2,
                        hidden=3072, n_heads=48, head_dim=64, ffn_dim=12288,
                        frames=13, height=30, width=45, n_text=226,
                        patch_h=2, patch_w=2, ratio=0.25, n_steps=2),
    # config 4: full 42-layer 5B-shaped DiT, 50-step schedule
    "cvx5b_42l": _cfg(name="cvx5b_42l", n_layers=42, n_shallow=8, interval=4,
                      hidden=3072, n_heads=48, head_dim=64, ffn_dim=12288,
                      frames=13, height=30, width=45, n_text=226,
                      patch_h=2, patch_w=2, ratio=0.25, n_steps=50),
    # config 5: long-video stress, one 5B-shaped block at 25 latent frames
    "cvx5b_long": _cfg(name="cvx5b_long", n_layers=2, n_shallow=1, interval=2,
                       hidden=3072, n_heads=48, head_dim=64, ffn_dim=12288,
                       frames=25, height=30, width=45, n_text=226,
                       patch_h=2, patch_w=2, ratio=0.25, n_steps=2),
    # structure-identical reduced instance of config 4 the oracle can finish
    "reduced_42l": _cfg(name="reduced_42l", n_layers=42, n_shallow=8, interval=4,
                        hidden=256, n_heads=4, head_dim=64, ffn_dim=1024,
                        frames=2, height=10, width=15, n_text=26,
                        patch_h=2, patch_w=2, ratio=0.25, n_steps=6),
    # the paper's own operating point (Sec. 4.1): 2x3 patches, R=0.2, K=20, M=2
    "paper_point": _cfg(name="paper_point", n_layers=42, n_shallow=20, interval=2,
                        hidden=3072, n_heads=48, head_dim=64, ffn_dim=12288,
                        frames=13, height=30, width=45, n_text=226,
                        patch_h=2, patch_w=3, ratio=0.2, n_steps=50),
}
# the other settings Sec. 4.1 names for that operating point: interval M = 3, and the 30-step schedule
CONFIGS["paper_point_m3"] = CONFIGS["paper_point"].with_(name="paper_point_m3", interval=3)
CONFIGS["paper_point_t30"] = CONFIGS["paper_point"].with_(name="paper_point_t30", n_steps=30)
CONFIGS["paper_point_m3_t30"] = CONFIGS["paper_point"].with_(name="paper_point_m3_t30", interval=3, n_steps=30)

# (patch_h, patch_w, ratio) for the refresh-ratio sweep of config 3
RATIO_SWEEP = {
    "10": dict(patch_h=2, patch_w=5, ratio=0.10),
    "25": dict(patch_h=2, patch_w=2, ratio=0.25),
    "50": dict(patch_h=2, patch_w=2, ratio=0.50),
}


def get_config(name: str, **overrides) -> HeroConfig:
    cfg = CONFIGS[name]
    return cfg.with_(**overrides) if overrides else cfg


# ----------------------------------------------------------------------------
# bf16 value handling of drawn inputs (round-to-nearest-even on the fp32 bits)
# ----------------------------------------------------------------------------

def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 array (exact widening)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is exactly representable in bf16."""
    return from_bf16_bits(bf16_bits(a)).reshape(np.shape(a))


# ----------------------------------------------------------------------------
# seeded draws
# ----------------------------------------------------------------------------

WEIGHT_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "ln2_g", "ln2_b", "w_ff1", "b_ff1", "w_ff2", "b_ff2")


def make_layer_weights(cfg: HeroConfig, layer: int, seed: int = 0,
                       std: float = 0.02, ln_affine_noise: float = 0.0
                       ) -> Dict[str, np.ndarray]:
    """Weights of one block, drawn N(0, std) and rounded to bf16 values.

    Linear weights use the [out_features, in_features] row-major layout.
    LayerNorm gain/bias are 1/0 unless ln_affine_noise > 0 (used by tests so a
    dropped gain or bias cannot hide).
    """
    rng = np.random.default_rng([seed, layer, 0xD17])
    d, f = cfg.hidden, cfg.ffn_dim

    def draw(*shape):
        return round_to_bf16((rng.standard_normal(shape, dtype=np.float32) * np.float32(std)))

    w = {
        "w_qkv": draw(3 * d, d), "b_qkv": draw(3 * d),
        "w_o": draw(d, d), "b_o": draw(d),
        "w_ff1": draw(f, d), "b_ff1": draw(f),
        "w_ff2": draw(d, f), "b_ff2": draw(d),
    }
    for nm in ("ln1", "ln2"):
        g = np.ones(d, np.float32)
        b = np.zeros(d, np.float32)
        if ln_affine_noise > 0:
            g = g + rng.standard_normal(d, dtype=np.float32) * np.float32(ln_affine_noise)
            b = b + rng.standard_normal(d, dtype=np.float32) * np.float32(ln_affine_noise)
        w[nm + "_g"] = round_to_bf16(g)
        w[nm + "_b"] = round_to_bf16(b)
    return w


BLOCK_ADALN, BLOCK_QKNORM, BLOCK_ROPE = 1, 2, 4
MOD_ROWS = ("shift1_v", "scale1_v", "gate1_v", "shift1_t", "scale1_t", "gate1_t",
            "shift2_v", "scale2_v", "gate2_v", "shift2_t", "scale2_t", "gate2_t")


def make_block_extras(cfg: HeroConfig, layer: int, seed: int = 0, step: int = 0, noise: float = 0.1
                      ) -> Dict[str, np.ndarray]:
    """Seeded draws of the extra parameters of the modulated block: per-head q/k
    LayerNorm gain/bias ([head_dim], 1/0 plus noise) and the modulation table
    "mod" [12, hidden] (rows as in MOD_ROWS; shift, scale ~ N(0, noise), gate ~
    1 + N(0, noise)), which depends on `step` the way a timestep embedding would.
    All values are bf16-representable.  Pure draws: no method arithmetic."""
    rng = np.random.default_rng([seed, layer, 0xADA])
    hd, d = cfg.head_dim, cfg.hidden
    out = {}
    for nm in ("qn", "kn"):
        out[nm + "_g"] = round_to_bf16(1 + rng.standard_normal(hd, dtype=np.float32) * np.float32(noise))
        out[nm + "_b"] = round_to_bf16(rng.standard_normal(hd, dtype=np.float32) * np.float32(noise))
    rs = np.random.default_rng([seed, layer, step, 0x30D])
    mod = rs.standard_normal((12, d), dtype=np.float32) * np.float32(noise)
    for i, nm in enumerate(MOD_ROWS):
        if nm.startswith("gate"):
            mod[i] += 1.0
    out["mod"] = round_to_bf16(mod)
    return out


def make_tokens(cfg: HeroConfig, seed: int = 1) -> np.ndarray:
    """Joint token sequence [N, hidden], N(0,1), bf16-representable fp32.

    Rows 0..n_text-1 are text tokens, then video token (t, y, x) sits at row
    n_text + (t*height + y)*width + x.
    """
    rng = np.random.default_rng([seed, 0x70C])
    return round_to_bf16(rng.standard_normal((cfg.n_tokens, cfg.hidden), dtype=np.float32))


def perturb_tokens(x: np.ndarray, seed: int = 2, std: float = 0.1) -> np.ndarray:
    """x + N(0, std): a neighbouring denoising step's input (adjacent steps are similar)."""
    rng = np.random.default_rng([seed, 0x9E7])
    return round_to_bf16(x + rng.standard_normal(x.shape, dtype=np.float32) * np.float32(std))


def euler_update(x_in, y_out, text0, n_text: int, n_steps: int):
    """Toy sampler update between denoising steps (harness-defined, not the paper's).

    v = y_video - x_video is the model's output (sum of the residual branches);
    x_video <- x_video - v / n_steps; text rows are reset to the original text
    tokens.  Works on numpy arrays and torch tensors alike.
    """
    nxt = x_in.copy() if hasattr(x_in, "copy") else x_in.clone()
    nxt[n_text:] = x_in[n_text:] - (y_out[n_text:] - x_in[n_text:]) / n_steps
    nxt[:n_text] = text0
    return nxt
