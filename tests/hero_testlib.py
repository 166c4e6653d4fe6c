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
        dev = {n: to_dev_bf16(w[n]) for n in WEIGHT_NAMES}
        # extra parameters of the modulated block, under the names the C struct uses
        for src, dst in (("qn_g", "q_norm_g"), ("qn_b", "q_norm_b"), ("kn_g", "k_norm_g"), ("kn_b", "k_norm_b"),
                         ("mod", "mod")):
            if src in w:
                dev[dst] = to_dev_bf16(w[src])
        cache.hero_set_layer_weights(l, dev)


def error_stats(got: np.ndarray, want: np.ndarray):
    diff = np.abs(got - want)
    return float(diff.max()), float(diff.sum() / max(np.abs(want).sum(), 1e-30))


def abs_bound(want: np.ndarray, max_abs: float) -> np.ndarray:
    """Per-element absolute bound: max_abs for |v| <= 1, max_abs * |v| beyond (2 % relative,
    about 5 bf16 ulps, continuous at 1).  bf16 errors are relative: a stored value in [4, 8)
    carries a half-ulp of up to 0.0156 on top of the error its bf16-rounded operands carry
    (sigma ~ 2e-3 .. 3e-3 per element after a 12288-deep FFN contraction), so a fixed 2e-2
    cannot hold over 10^5 .. 10^8 compared elements for any bf16 pipeline; a numpy emulation of
    the bf16 chain shows the same worst case as the GPU."""
    return max_abs * np.maximum(1.0, np.abs(want))


def assert_close(got, want, what="", max_abs=MAX_ABS_TOL, mean_rel=MEAN_REL_TOL, stored_parts=None):
    """stored_parts: arrays of intermediates that the pipeline stores in bf16 on the way to `want`
    (e.g. the attention feature that is later summed with the FFN feature).  The per-element
    bound then scales with the largest magnitude among `want` and those parts: a sum of 0.4 that
    was formed from a stored 2.1 and a -1.7 carries the rounding of the 2.1."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    ma, mr = error_stats(got, want)
    mag = np.abs(want)
    for part in (stored_parts or ()):
        mag = np.maximum(mag, np.abs(np.asarray(part, np.float64)))
    worst = float((np.abs(got - want) - abs_bound(mag, max_abs)).max())
    assert worst <= 0.0 and mr <= mean_rel, \
        f"{what}: max-abs {ma:.3e} (tol {max_abs}, scaled by |v| above 1; exceeded by {worst:.3e}), " \
        f"mean-rel {mr:.3e} (tol {mean_rel})"
    return ma, mr
