"""Pins for the oracle's block components (CPU only).

Each routine is checked against something other than itself: a library routine
(torch CPU), brute-force python loops, closed forms and special cases.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import hero_oracle as O


def rng(seed):
    return np.random.default_rng(seed)


def test_layer_norm_matches_library_and_closed_form():
    r = rng(0)
    x = r.standard_normal((7, 96)) * 3 + 1.5
    g = r.standard_normal(96)
    b = r.standard_normal(96)
    ref = F.layer_norm(torch.from_numpy(x), (96,), torch.from_numpy(g), torch.from_numpy(b), 1e-5).numpy()
    np.testing.assert_allclose(O.layer_norm(x, g, b, 1e-5), ref, rtol=1e-12, atol=1e-12)
    # closed form: unit gain, zero bias -> zero mean, variance var/(var+eps)
    y = O.layer_norm(x, np.ones(96), np.zeros(96), 1e-5)
    np.testing.assert_allclose(y.mean(-1), 0, atol=1e-13)
    v = x.var(-1)
    np.testing.assert_allclose(y.var(-1), v / (v + 1e-5), rtol=1e-12)
    # invariance: shifting and scaling the input row leaves LN unchanged up to eps
    y2 = O.layer_norm(x * 7.0 + 3.0, np.ones(96), np.zeros(96), 0.0)
    y3 = O.layer_norm(x, np.ones(96), np.zeros(96), 0.0)
    np.testing.assert_allclose(y2, y3, rtol=1e-10, atol=1e-10)


def test_gelu_tanh_matches_library_and_limits():
    x = np.linspace(-6, 6, 1001)
    ref = F.gelu(torch.from_numpy(x), approximate="tanh").numpy()
    np.testing.assert_allclose(O.gelu_tanh(x), ref, rtol=1e-12, atol=1e-14)
    assert O.gelu_tanh(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.gelu_tanh(np.array([10.0])), [10.0], rtol=1e-12)
    np.testing.assert_allclose(O.gelu_tanh(np.array([-10.0])), [0.0], atol=1e-12)
    # within 1e-3 of the erf definition x * Phi(x)
    erf_form = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x])
    assert np.abs(O.gelu_tanh(x) - erf_form).max() < 1e-3


def test_linear_matches_library_and_catches_transpose():
    r = rng(1)
    x = r.standard_normal((5, 12))
    w = r.standard_normal((9, 12))   # [out, in]
    b = r.standard_normal(9)
    ref = F.linear(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(b)).numpy()
    np.testing.assert_allclose(O.linear(x, w, b), ref, rtol=1e-12, atol=1e-12)
    # brute force
    for i in range(5):
        for o in range(9):
            assert abs(O.linear(x, w, b)[i, o] - (sum(x[i, c] * w[o, c] for c in range(12)) + b[o])) < 1e-12


def brute_attention(q, k, v, n_heads):
    r, d = q.shape
    n = k.shape[0]
    hd = d // n_heads
    out = np.zeros((r, d))
    for h in range(n_heads):
        for i in range(r):
            s = [sum(q[i, h * hd + c] * k[j, h * hd + c] for c in range(hd)) / math.sqrt(hd) for j in range(n)]
            m = max(s)
            e = [math.exp(t - m) for t in s]
            z = sum(e)
            for c in range(hd):
                out[i, h * hd + c] = sum(e[j] / z * v[j, h * hd + c] for j in range(n))
    return out


@pytest.mark.parametrize("case", ["plain", "peaky", "outlier"])
def test_attention_brute_force(case):
    r = rng(2)
    q = r.standard_normal((5, 16))
    k = r.standard_normal((11, 16))
    v = r.standard_normal((11, 16))
    if case == "peaky":
        q, k = q * 10, k * 10
    if case == "outlier":
        k[3] *= 100
    got = O.attention(q, k, v, 2)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, brute_attention(q, k, v, 2), rtol=1e-10, atol=1e-12)


def test_attention_matches_library_sdpa():
    r = rng(3)
    H, hd, n, m = 3, 8, 37, 13
    q = r.standard_normal((m, H * hd))
    k = r.standard_normal((n, H * hd))
    v = r.standard_normal((n, H * hd))
    tq = torch.from_numpy(q).view(m, H, hd).transpose(0, 1)
    tk = torch.from_numpy(k).view(n, H, hd).transpose(0, 1)
    tv = torch.from_numpy(v).view(n, H, hd).transpose(0, 1)
    ref = F.scaled_dot_product_attention(tq, tk, tv).transpose(0, 1).reshape(m, H * hd).numpy()
    np.testing.assert_allclose(O.attention(q, k, v, H), ref, rtol=1e-10, atol=1e-12)


def test_attention_special_cases():
    r = rng(4)
    k = r.standard_normal((9, 8))
    v = r.standard_normal((9, 8))
    # zero queries -> uniform weights -> mean of V
    out = O.attention(np.zeros((3, 8)), k, v, 2)
    np.testing.assert_allclose(out, np.tile(v.mean(0), (3, 1)), rtol=1e-12)
    # one key -> output is that key's value whatever the query
    out = O.attention(r.standard_normal((4, 8)), k[:1], v[:1], 2)
    np.testing.assert_allclose(out, np.tile(v[0], (4, 1)), rtol=1e-12)
    # permuting the keys (with their values) changes nothing
    q = r.standard_normal((4, 8))
    perm = r.permutation(9)
    np.testing.assert_allclose(O.attention(q, k, v, 2), O.attention(q, k[perm], v[perm], 2), rtol=1e-10, atol=1e-12)
    # heads are independent: changing head 1's keys leaves head 0's output alone
    k2 = k.copy()
    k2[:, 4:] += 1.0
    np.testing.assert_array_equal(O.attention(q, k, v, 2)[:, :4], O.attention(q, k2, v, 2)[:, :4])


def test_ffn_matches_library():
    r = rng(5)
    d, f = 12, 20
    u = r.standard_normal((6, d))
    w = {"w_ff1": r.standard_normal((f, d)), "b_ff1": r.standard_normal(f),
         "w_ff2": r.standard_normal((d, f)), "b_ff2": r.standard_normal(d)}
    t = lambda a: torch.from_numpy(a)
    ref = F.linear(F.gelu(F.linear(t(u), t(w["w_ff1"]), t(w["b_ff1"])), approximate="tanh"),
                   t(w["w_ff2"]), t(w["b_ff2"])).numpy()
    np.testing.assert_allclose(O.ffn(u, w), ref, rtol=1e-11, atol=1e-12)


def test_block_forward_matches_library_block():
    """Eq. 2 assembled from torch CPU routines (pre-LN, biased linears, tanh GELU)."""
    from workloads import get_config, make_layer_weights, make_tokens
    cfg = get_config("tiny")
    w = make_layer_weights(cfg, 0, seed=0, std=0.2, ln_affine_noise=0.3)
    x = make_tokens(cfg, seed=1).astype(np.float64)[:50]
    w64 = {k: v.astype(np.float64) for k, v in w.items()}
    y, g_attn, g_ffn, k, v = O.block_forward(x, w64, cfg.n_heads, cfg.ln_eps)

    t = {k_: torch.from_numpy(v_) for k_, v_ in w64.items()}
    tx = torch.from_numpy(x)
    d, H, hd = cfg.hidden, cfg.n_heads, cfg.head_dim
    u = F.layer_norm(tx, (d,), t["ln1_g"], t["ln1_b"], cfg.ln_eps)
    qkv = F.linear(u, t["w_qkv"], t["b_qkv"])
    q_, k_, v_ = qkv.split(d, dim=1)
    sh = lambda a: a.view(-1, H, hd).transpose(0, 1)
    o = F.scaled_dot_product_attention(sh(q_), sh(k_), sh(v_)).transpose(0, 1).reshape(-1, d)
    ga = F.linear(o, t["w_o"], t["b_o"])
    a = tx + ga
    gf = F.linear(F.gelu(F.linear(F.layer_norm(a, (d,), t["ln2_g"], t["ln2_b"], cfg.ln_eps),
                                  t["w_ff1"], t["b_ff1"]), approximate="tanh"), t["w_ff2"], t["b_ff2"])
    np.testing.assert_allclose(g_attn, ga.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(g_ffn, gf.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(y, (a + gf).numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(k, k_.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(v, v_.numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- stability score (Sec. 3.2)

def test_second_difference_variance_closed_forms():
    rng = np.random.default_rng(3)
    a, b, c = rng.standard_normal((3, 40, 16))
    # linear in time: second differences vanish
    lin = [a + b * t for t in range(5)]
    assert O.second_difference_variance(lin) < 1e-24
    # quadratic in time: D = 2c at every step, so the variance is Var(2c) over the elements
    quad = [a + b * t + c * t * t for t in range(6)]
    np.testing.assert_allclose(O.second_difference_variance(quad), np.var(2.0 * c), rtol=1e-10)
    # the same quadratic with one coefficient for all elements: D is constant, variance 0
    quad1 = [a + b * t + 0.7 * t * t for t in range(4)]
    assert O.second_difference_variance(quad1) < 1e-20
    # hand-computed: features 0, 1, 4, 4 on two elements (second element doubled)
    f = [np.array([0.0, 0.0]), np.array([1.0, 2.0]), np.array([4.0, 8.0]), np.array([4.0, 8.0])]
    # D_1 = (2, 4), D_2 = (-3, -6): mean -0.75, variance = mean of squares - mean^2
    d = np.array([2.0, 4.0, -3.0, -6.0])
    np.testing.assert_allclose(O.second_difference_variance(f), np.mean(d * d) - d.mean() ** 2, rtol=1e-12)
    with pytest.raises(ValueError):
        O.second_difference_variance(f[:2])


def test_second_difference_variance_of_white_noise_is_six_sigma_squared():
    rng = np.random.default_rng(4)
    sigma = 0.3
    feats = [sigma * rng.standard_normal(200000) for _ in range(3)]
    # Var(F2 - 2 F1 + F0) = (1 + 4 + 1) sigma^2 for independent steps
    np.testing.assert_allclose(O.second_difference_variance(feats), 6 * sigma ** 2, rtol=0.02)


def test_stability_scores_normalise_and_invert():
    s = O.stability_scores([4.0, 1.0, 2.5, 1.0])
    np.testing.assert_allclose(s, [0.0, 1.0, 0.5, 1.0])
    np.testing.assert_allclose(O.stability_scores([3.0, 3.0]), [1.0, 1.0])
    assert s.min() == 0.0 and s.max() == 1.0
