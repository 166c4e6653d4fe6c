"""Shared helpers of the GPU parity tests (uploading seeded inputs, tolerances)."""
import os

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


def bf16_half_ulp(mag: np.ndarray) -> np.ndarray:
    """Half a unit in the last place of bf16 (8 significant bits) at magnitude `mag`: 2^(e-8) for
    mag in [2^e, 2^(e+1))."""
    mag = np.maximum(np.abs(np.asarray(mag, np.float64)), 2.0 ** -126)
    return np.exp2(np.floor(np.log2(mag)) - 8.0)


FLAT_HALF_ULP = 2.0 ** -7     # half-ulp of the binade [2, 4): the largest one the flat tolerance has to absorb


def abs_bound(want: np.ndarray, max_abs: float, stored_parts=()) -> np.ndarray:
    """Per-element absolute bound without an ideal-pipeline reference at hand.  The flat tolerance
    `max_abs` covers the arithmetic error and one bf16 storage rounding of a value below 4 in
    magnitude (half-ulp <= 2^-7).  A value stored at |v| in [4, 8) carries a half-ulp of
    2^-6 = 0.0156 (0.031 in [8, 16), ...) whatever computed it: the bound grows by what that
    exceeds 2^-7.  Every further tensor that the pipeline stores in bf16 on the way
    (`stored_parts`: the attention feature that is later summed with the FFN feature; K before
    its normalisation and rotation in the modulated block) adds its own half-ulp.
    tests/test_bf16_error_budget.py derives this on the CPU: the oracle's own routines with one
    bf16 rounding per stored tensor exceed the flat 2e-2 for K and V exactly where this bound
    gives way, and stay inside it."""
    extra = np.maximum(0.0, bf16_half_ulp(want) - FLAT_HALF_ULP)
    for t in stored_parts:
        extra = extra + bf16_half_ulp(t)
    return max_abs + extra


MAG_BINS = (0.0, 1.0, 2.0, 4.0, 8.0, np.inf)      # |oracle value|: one bf16 binade per bin from 1 on


def _log(line):
    path = os.environ.get("HERO_PARITY_LOG")
    if path:
        with open(path, "a") as f:
            f.write(line + "\n")


def assert_close(got, want, what="", max_abs=MAX_ABS_TOL, mean_rel=MEAN_REL_TOL, stored_parts=None, emul=None):
    """The parity gate for bf16 activations against the float64 oracle `want`.

    Always: the aggregate relative error sum|got - want| / sum|want| <= mean_rel.

    Without `emul`: every element within abs_bound(...) -- the flat `max_abs` below |v| = 4.

    With `emul` -- the same quantity from the oracle's routines with one bf16 rounding per stored
    tensor (tests/block_oracle.py, stored_bf16=True; CPU values only, an ideal bf16 pipeline):
    on a feature of rms 1.6 behind a 12288-deep contraction of rounded activations that ideal
    pipeline itself sits at sigma ~ 4e-3 and leaves the flat tolerance on thousands of 10^7
    elements, at every magnitude (tests/test_bf16_error_budget.py), and its rounding flips cascade
    differently for any other order of additions, so no per-element bound separates "bf16" from
    "wrong".  The gate is then that the GPU is no worse than the ideal pipeline: in every
    magnitude bin the number of elements beyond the flat tolerance is at most the ideal
    pipeline's (+25 % and counting noise), and the largest error is at most 1.3 x the ideal
    pipeline's (or the flat tolerance).

    Every call reports the raw max-abs error and the number of elements above the flat tolerance
    (in the failure message, and as a line in $HERO_PARITY_LOG when that is set)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    ma, mr = error_stats(got, want)
    err = np.abs(got - want)
    n_flat = int((err > max_abs).sum())
    parts = [np.asarray(p_, np.float64) for p_ in (stored_parts or ())]
    n_over = int((err > abs_bound(want, max_abs, parts)).sum())
    msg = (f"{what}: n={got.size} max-abs {ma:.3e}, {n_flat} above the flat {max_abs:g}, {n_over} above the "
           f"per-element bound, mean-rel {mr:.3e} (tol {mean_rel:g})")
    if emul is None:
        _log(msg)
        assert n_over == 0 and mr <= mean_rel, msg
        return ma, mr
    e_err = np.abs(np.asarray(emul, np.float64) - want)
    e_ma = float(e_err.max())
    mag = np.abs(want)
    ok = mr <= mean_rel and ma <= max(max_abs, 1.3 * e_ma)
    bins = []
    for lo, hi in zip(MAG_BINS[:-1], MAG_BINS[1:]):
        m = (mag >= lo) & (mag < hi)
        g, e = int((err[m] > max_abs).sum()), int((e_err[m] > max_abs).sum())
        bins.append(f"[{lo:g},{hi:g}) {g}/{e}")
        ok = ok and g <= 1.25 * e + 3.0 * np.sqrt(e) + 5
    msg += (f"; ideal bf16 pipeline: max-abs {e_ma:.3e}, {int((e_err > max_abs).sum())} above the flat tolerance; "
            f"above it per |v| bin (gpu/ideal): " + ", ".join(bins))
    _log(msg)
    assert ok, msg
    return ma, mr
