"""Where the parity tolerance comes from -- derived on the CPU alone, no GPU value anywhere.

The contract is max-abs 2e-2 / mean-relative 5e-3 against the float64 oracle.  A pipeline with bf16
operands and bf16-stored tensors cannot hold a flat 2e-2 everywhere, whoever writes it:
  * a value stored at |v| in [4, 8) is off by up to half a bf16 ulp = 2^-6 = 0.0156 before any
    arithmetic error is added (0.031 in [8, 16), ...);
  * a contraction over k rounded operands leaves a Gaussian-like error of
    sigma ~ 2^-8 / sqrt(3) * 0.72 * sqrt(sum a_i^2 w_i^2): 1.8e-3 on a K projection of rms 1.1,
    4e-3 on the 5B-shaped block's feature sum (rms 1.6, after a 12288-deep contraction), so that
    2e-2 is 11 sigma for K but only 5 sigma for the feature sum, and a comparison of 10^7 elements
    meets the 5-sigma tail.
This file runs the oracle's own routines twice on a 5B-shaped block (3072 wide, 48 heads, FFN
12288; 1024 tokens) -- once exact, once with one bf16 rounding per stored tensor
(tests/block_oracle.py) -- and shows that
  1. K and V of the ideal bf16 pipeline leave the flat 2e-2 only at |v| >= 4, and stay inside
     hero_testlib.abs_bound (flat 2e-2 below 4, plus the excess half-ulp beyond), which is tight;
  2. the feature sum S of the ideal pipeline leaves the flat 2e-2 at small magnitudes as well, at
     the rate its sigma predicts -- which is why the full-size GPU tests of S take the ideal
     pipeline as a second reference (the GPU must leave the flat 2e-2 no more often than the
     ideal pipeline does, bin by bin of |v|, and no further) instead of a widened flat bound;
  3. with features of rms ~0.3 (weights at half the scale) the ideal pipeline meets the flat
     2e-2 everywhere: the refinements vanish where the contract can be met as written.
"""
import math

import numpy as np
import pytest

from workloads import get_config, make_layer_weights, make_tokens, round_to_bf16
from block_oracle import BlockOracle, r16
from hero_testlib import MAX_ABS_TOL, abs_bound, bf16_half_ulp

CFG = get_config("cvx5b_block").with_(frames=1, height=30, width=32, n_text=64)     # 1024 tokens


def block_pair(std):
    """(exact, ideal-bf16) -> dicts with K, V, g_attn, S of every row of one 5B-shaped block."""
    w = make_layer_weights(CFG, 0, seed=0, std=std)
    x = make_tokens(CFG, seed=1).astype(np.float64)
    rows = np.arange(CFG.n_tokens)
    out = []
    for stored in (False, True):
        orc = BlockOracle(CFG, w, stored_bf16=stored)
        k, v = orc.kv(x, rows)
        ga, gf, s = orc.rows(x, rows, k, v)
        out.append(dict(k=k, v=v, ga=ga, s=s))
    return out


@pytest.fixture(scope="module")
def pair():
    return block_pair(0.02)


def test_half_ulp_helper_bounds_the_rounding_error():
    rng = np.random.default_rng(0)
    v = rng.standard_normal(200000) * np.exp2(rng.integers(-6, 5, 200000))
    err = np.abs(r16(v) - v)
    hu = bf16_half_ulp(v)
    assert (err <= hu * (1 + 2.0 ** -14)).all()          # (r16 passes through fp32: 2^-24 relative on top)
    assert (err > 0.98 * hu).any()                      # and it is attained
    np.testing.assert_array_equal(bf16_half_ulp([1.0, 1.99, 2.0, 3.99, 4.0, 8.0]), [2.0 ** -8, 2.0 ** -8, 2.0 ** -7, 2.0 ** -7, 2.0 ** -6, 2.0 ** -5])


def test_k_and_v_of_the_ideal_bf16_pipeline_leave_the_flat_tolerance_only_beyond_4(pair):
    exact, ideal = pair
    for name in ("k+v",):                               # one projection: pooled, 6.3 M elements
        want, got = np.concatenate([exact["k"], exact["v"]]), np.concatenate([ideal["k"], ideal["v"]])
        err, mag = np.abs(got - want), np.abs(want)
        beyond = err > MAX_ABS_TOL
        assert beyond.any(), f"{name}: the ideal pipeline was expected to exceed the flat tolerance somewhere"
        assert mag[beyond].min() >= 4.0, f"{name}: flat tolerance exceeded at |v| = {mag[beyond].min():.3f}"
        bound = abs_bound(want, MAX_ABS_TOL)
        assert (err <= bound).all(), f"{name}: ideal pipeline outside abs_bound by {(err - bound).max():.3e}"
        # tight: the ideal pipeline uses most of the bound on both sides of |v| = 4
        lo, hi = mag < 4.0, mag >= 4.0
        assert (err[lo] / bound[lo]).max() > 0.7 and (err[hi] / bound[hi]).max() > 0.7
        # error model: two roundings (operands, result), each of relative rms 2^-8/sqrt(3) * 0.72
        sigma = math.sqrt(2.0) * (2.0 ** -8 / math.sqrt(3.0)) * 0.72 * math.sqrt((want ** 2).mean())
        rms = math.sqrt((err ** 2).mean())
        assert 0.8 * sigma < rms < 1.25 * sigma, (rms, sigma)


def test_feature_sum_of_the_ideal_bf16_pipeline_leaves_the_flat_tolerance_at_every_magnitude(pair):
    exact, ideal = pair
    want, got = exact["s"], ideal["s"]
    err, mag = np.abs(got - want), np.abs(want)
    small = mag < 0.5                                    # storage half-ulp <= 0.001: the error is all operand rounding
    sigma_up = math.sqrt((err[small] ** 2).mean())
    rms_s = math.sqrt((want ** 2).mean())
    assert 1.4 < rms_s < 1.9 and 3.2e-3 < sigma_up < 4.8e-3, (rms_s, sigma_up)
    assert MAX_ABS_TOL / sigma_up < 5.6                 # 10^7 elements hold ~ 10^7 * P(|z| > 5.6) = 0.2 .. 6 beyond it
    # exceedances at small magnitudes, where no half-ulp argument applies ...
    assert (err[mag < 2.0] > MAX_ABS_TOL).sum() >= 1
    # ... at about the Gaussian rate (3.1 M elements, two-sided tail beyond 2e-2 / sigma)
    z = MAX_ABS_TOL / sigma_up
    expect = small.sum() * math.erfc(z / math.sqrt(2.0))
    seen = (err[small] > MAX_ABS_TOL).sum()
    assert seen <= 10 * expect + 5, (seen, expect)
    # and the bulk of them where the stored value's own half-ulp is 0.0156
    assert (err[mag >= 4.0] > MAX_ABS_TOL).mean() > 50 * (err[mag < 4.0] > MAX_ABS_TOL).mean()
    # the mean-relative criterion is met with room: it is the sharp one
    assert err.sum() / mag.sum() < 0.6 * 5e-3
    # the attention feature on its own is small here and nowhere near the tolerance
    assert np.abs(ideal["ga"] - exact["ga"]).max() < 0.25 * MAX_ABS_TOL


def test_at_small_feature_scale_the_ideal_bf16_pipeline_meets_the_flat_tolerance():
    exact, ideal = block_pair(0.01)
    for name in ("k", "v", "s"):
        err = np.abs(ideal[name] - exact[name])
        assert err.max() < MAX_ABS_TOL, (name, err.max())
        assert (abs_bound(exact[name], MAX_ABS_TOL) == MAX_ABS_TOL).all()


@pytest.mark.parametrize("flags", [0, 7])
def test_block_oracle_in_exact_mode_is_the_oracles_block(flags):
    """tests/block_oracle.py assembles the block from the oracle's routines row by row; in exact mode
    it must reproduce the oracle's own full layer (plain block: Eq. 2 as block_forward; modulated
    block: HeroOracle.full_layer), so that its bf16 mode differs from the oracle by the roundings only."""
    from oracle import hero_oracle as O
    from workloads import make_block_extras
    cfg = get_config("tiny").with_(n_layers=1, n_shallow=1, hidden=256, n_heads=4, head_dim=64, ffn_dim=512,
                                   frames=2, height=6, width=7, n_text=9, block_flags=flags)
    w = make_layer_weights(cfg, 0, seed=3, std=0.05, ln_affine_noise=0.1)
    if flags:
        w.update(make_block_extras(cfg, 0, seed=3, step=0))
    x = make_tokens(cfg, seed=4).astype(np.float64)
    orc = O.HeroOracle(cfg, [w])
    y = orc.full_layer(0, x)
    c = orc.caches[0]
    bo = BlockOracle(cfg, w)
    rows = np.arange(cfg.n_tokens)
    k, v = bo.kv(x, rows)
    np.testing.assert_allclose(k, c.k, rtol=0, atol=1e-12)
    np.testing.assert_allclose(v, c.v, rtol=0, atol=1e-12)
    pick = np.array([0, 8, 9, 40, cfg.n_tokens - 1])
    ga, gf, s = bo.rows(x[pick], pick, k, v)
    np.testing.assert_allclose(ga, c.g_attn[pick], rtol=0, atol=1e-12)
    np.testing.assert_allclose(gf, c.g_ffn[pick], rtol=0, atol=1e-12)
    np.testing.assert_allclose(x[pick] + s, y[pick], rtol=0, atol=1e-12)
    # and the bf16 mode stays within a few bf16 ulps of it
    ga16, gf16, s16 = BlockOracle(cfg, w, stored_bf16=True).rows(x[pick], pick, *BlockOracle(cfg, w, stored_bf16=True).kv(x, rows))
    assert 0 < np.abs(s16 - s).max() < 0.05
