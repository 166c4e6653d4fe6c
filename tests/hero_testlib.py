"""Shared helpers of the GPU parity tests (uploading seeded inputs, tolerances)."""
import numpy as np
import torch

from workloads import bf16_bits, from_bf16_bits, make_layer_weights, WEIGHT_NAMES

MAX_ABS_TOL = 2e-2     # bf16 activations: max |gpu - oracle|
MEAN_REL_TOL = 5e-3    # sum |gpu - oracle| / sum |oracle|


def to_dev_bf16(a: np.ndarray) -> torch.Tensor:
    """bf16-representable fp32 numpy array -> bf16 device tensor, bit-exact."""
    bits = bf16_bits(np.asarray(a, np.float32)).astype(np.int16).reshape(np.shape(a))
    return torch.from_numpy(bits).cuda().view(torch.bfloat16)


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def upload_weights(cache, cfg, weights):
    for l, w in enumerate(weights):
        cache.hero_set_layer_weights(l, {n: to_dev_bf16(w[n]) for n in WEIGHT_NAMES})


def error_stats(got: np.ndarray, want: np.ndarray):
    diff = np.abs(got - want)
    return float(diff.max()), float(diff.sum() / max(np.abs(want).sum(), 1e-30))


def assert_close(got, want, what="", max_abs=MAX_ABS_TOL, mean_rel=MEAN_REL_TOL):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    ma, mr = error_stats(got, want)
    assert ma <= max_abs and mr <= mean_rel, f"{what}: max-abs {ma:.3e} (tol {max_abs}), mean-rel {mr:.3e} (tol {mean_rel})"
    return ma, mr
