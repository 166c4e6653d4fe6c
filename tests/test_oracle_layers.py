"""Pins for the oracle's layer operations and step schedule (CPU only).

  P1  refresh with idx = all rows reproduces the full block forward
  P2  extrapolation is exact on features linear in the step; k=0 and equal
      generations reduce to reuse
  P4  locality: untouched cache rows are bit-unchanged, refreshed rows equal the
      full forward's rows when only those rows' inputs changed
  P5  degenerate schedules: empty selection = pure reuse; K=0 = forecasting on
      every layer; K=L with all rows = all-full compute
"""
import numpy as np
import pytest

from oracle import hero_oracle as O
from workloads import get_config, make_layer_weights, make_tokens, perturb_tokens, euler_update


def setup(cfg, std=0.2, n_layers=None):
    L = n_layers or cfg.n_layers
    ws = [make_layer_weights(cfg, l, seed=0, std=std, ln_affine_noise=0.2) for l in range(L)]
    x = make_tokens(cfg, seed=1).astype(np.float64)
    return ws, x


def test_p1_refresh_all_rows_equals_full_forward():
    cfg = get_config("tiny", n_layers=1, n_shallow=1)
    ws, x0 = setup(cfg)
    orc = O.HeroOracle(cfg, ws)
    orc.full_layer(0, perturb_tokens(x0.astype(np.float32), seed=2, std=0.5).astype(np.float64))  # stale fill
    x1 = x0
    y_ref, g_attn, g_ffn, k, v = O.block_forward(x1, orc.w[0], cfg.n_heads, cfg.ln_eps)
    idx = np.random.default_rng(0).permutation(cfg.n_tokens)   # all rows, any order
    y = orc.refresh_layer(0, x1, idx)
    c = orc.caches[0]
    np.testing.assert_allclose(y, y_ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(c.g_attn, g_attn, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(c.g_ffn, g_ffn, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(c.k, k, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(c.v, v, rtol=1e-12, atol=1e-13)


def test_p1b_video_only_full_ratio_matches_full_forward_on_video_rows():
    """100 % of video rows refreshed, text bypassed: video rows of G equal the full
    forward's when the text inputs have not changed since the fill."""
    cfg = get_config("tiny", n_layers=1, n_shallow=1)
    ws, x0 = setup(cfg)
    orc = O.HeroOracle(cfg, ws)
    orc.full_layer(0, x0)
    x1 = x0.copy()
    x1[cfg.n_text:] = perturb_tokens(x0.astype(np.float32), 3, 0.3).astype(np.float64)[cfg.n_text:]
    _, g_attn, g_ffn, _, _ = O.block_forward(x1, orc.w[0], cfg.n_heads, cfg.ln_eps)
    text_before = orc.caches[0].g_attn[:cfg.n_text].copy()
    orc.refresh_layer(0, x1, np.arange(cfg.n_text, cfg.n_tokens))
    c = orc.caches[0]
    np.testing.assert_allclose(c.g_attn[cfg.n_text:], g_attn[cfg.n_text:], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(c.g_ffn[cfg.n_text:], g_ffn[cfg.n_text:], rtol=1e-10, atol=1e-12)
    np.testing.assert_array_equal(c.g_attn[:cfg.n_text], text_before)


def test_p2_extrapolation_closed_form():
    r = np.random.default_rng(1)
    a, b = r.standard_normal((6, 5)), r.standard_normal((6, 5))
    M = 4
    # features linear in the step s: G(s) = a + b*s; full steps at s=4 and s=8 (prev, cur)
    g = lambda s: a + b * s
    for k in range(0, M + 1):
        np.testing.assert_allclose(O.extrapolated(g(8), g(4), k, M), g(8 + k), rtol=1e-13, atol=1e-13)
    # k = 0 -> reuse, equal generations -> reuse, no previous generation -> reuse
    np.testing.assert_array_equal(O.extrapolated(g(8), g(4), 0, M), g(8))
    np.testing.assert_array_equal(O.extrapolated(g(8), g(8), 3, M), g(8))
    np.testing.assert_array_equal(O.extrapolated(g(8), None, 3, M), g(8))
    # sign pin: a feature that grew keeps growing
    assert (O.extrapolated(np.ones(3) * 2, np.ones(3), 1, 2) == 2.5).all()


def test_p2_extrapolate_layer_adds_both_branches():
    cfg = get_config("tiny")
    c = O.LayerCache()
    r = np.random.default_rng(2)
    c.g_attn, c.g_attn_prev = r.standard_normal((4, 3)), r.standard_normal((4, 3))
    c.g_ffn, c.g_ffn_prev = r.standard_normal((4, 3)), r.standard_normal((4, 3))
    x = r.standard_normal((4, 3))
    k, M = 3, 4
    want = x + (c.g_attn + (c.g_attn - c.g_attn_prev) * 0.75) + (c.g_ffn + (c.g_ffn - c.g_ffn_prev) * 0.75)
    np.testing.assert_allclose(O.extrapolate_layer(x, c, k, M), want, rtol=1e-13)


def test_p4_locality():
    cfg = get_config("tiny", n_layers=1, n_shallow=1)
    ws, x0 = setup(cfg)
    orc = O.HeroOracle(cfg, ws)
    orc.full_layer(0, x0)
    before = {n: getattr(orc.caches[0], n).copy() for n in ("g_attn", "g_ffn", "k", "v")}
    idx = np.array([20, 33, 100, 271, 16])
    x1 = x0.copy()
    x1[idx] += np.random.default_rng(3).standard_normal((len(idx), cfg.hidden)) * 0.5
    y = orc.refresh_layer(0, x1, idx)
    c = orc.caches[0]
    rest = np.setdiff1d(np.arange(cfg.n_tokens), idx)
    for n in ("g_attn", "g_ffn", "k", "v"):
        np.testing.assert_array_equal(getattr(c, n)[rest], before[n][rest])
        assert not np.array_equal(getattr(c, n)[idx], before[n][idx])
    # only rows idx changed since the fill -> refreshed rows equal the full forward's rows
    y_ref, g_attn, g_ffn, k, v = O.block_forward(x1, orc.w[0], cfg.n_heads, cfg.ln_eps)
    np.testing.assert_allclose(c.g_attn[idx], g_attn[idx], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(c.g_ffn[idx], g_ffn[idx], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(c.k[idx], k[idx], rtol=1e-12)
    np.testing.assert_allclose(y[idx], y_ref[idx], rtol=1e-10, atol=1e-12)
    # the other rows got x + cached features
    np.testing.assert_allclose(y[rest], x1[rest] + before["g_attn"][rest] + before["g_ffn"][rest], rtol=1e-13)


def test_p4_refreshed_queries_see_refreshed_keys():
    """K/V rows are written back before attention: a refreshed row's own new key is
    among the keys it attends to (otherwise P1 could not hold)."""
    cfg = get_config("tiny", n_layers=1, n_shallow=1)
    ws, x0 = setup(cfg, std=0.5)
    orc = O.HeroOracle(cfg, ws)
    orc.full_layer(0, x0)
    idx = np.array([40])
    x1 = x0.copy()
    x1[40] *= -3.0
    orc.refresh_layer(0, x1, idx)
    w = orc.w[0]
    d = cfg.hidden
    u = O.layer_norm(x1[idx], w["ln1_g"], w["ln1_b"], cfg.ln_eps)
    qkv = O.linear(u, w["w_qkv"], w["b_qkv"])
    np.testing.assert_allclose(orc.caches[0].k[40], qkv[0, d:2 * d], rtol=1e-12)
    np.testing.assert_allclose(orc.caches[0].v[40], qkv[0, 2 * d:], rtol=1e-12)
    g = O.linear(O.attention(qkv[:, :d], orc.caches[0].k, orc.caches[0].v, cfg.n_heads), w["w_o"], w["b_o"])
    np.testing.assert_allclose(orc.caches[0].g_attn[40], g[0], rtol=1e-10, atol=1e-12)


def test_p5_empty_selection_is_pure_reuse():
    cfg = get_config("tiny", n_layers=1, n_shallow=1)
    ws, x0 = setup(cfg)
    orc = O.HeroOracle(cfg, ws)
    orc.full_layer(0, x0)
    c = orc.caches[0]
    x1 = perturb_tokens(x0.astype(np.float32), 5, 0.2).astype(np.float64)
    y = orc.refresh_layer(0, x1, np.zeros(0, np.int32))
    np.testing.assert_array_equal(y, x1 + c.g_attn + c.g_ffn)


def run_schedule(cfg, ws, x0, n_steps):
    orc = O.HeroOracle(cfg, ws)
    x = x0.copy()
    text0 = x0[:cfg.n_text].copy()
    outs = []
    for s in range(n_steps):
        y = orc.step(x, s)
        outs.append(y)
        x = euler_update(x, y, text0, cfg.n_text, n_steps)
    return orc, outs


def test_p5_all_shallow_all_rows_is_all_full():
    """K = L and ratio 1 on video rows: cached steps differ from full steps only
    through the text rows' reuse; with M = 1 every step is full."""
    cfg = get_config("tiny", interval=1)
    ws, x0 = setup(cfg)
    orc, outs = run_schedule(cfg, ws, x0, 3)
    x = x0.copy()
    text0 = x0[:cfg.n_text].copy()
    for s in range(3):
        y = x
        for l in range(cfg.n_layers):
            y = O.block_forward(y, orc.w[l], cfg.n_heads, cfg.ln_eps)[0]
        np.testing.assert_allclose(outs[s], y, rtol=1e-10, atol=1e-12)
        x = euler_update(x, y, text0, cfg.n_text, 3)


def test_p5_k0_is_first_order_forecast_on_every_layer():
    cfg = get_config("tiny", n_shallow=0, interval=2)
    ws, x0 = setup(cfg)
    orc = O.HeroOracle(cfg, ws)
    text0 = x0[:cfg.n_text].copy()
    x = x0.copy()
    gens = []
    for s in range(4):
        y = orc.step(x, s)
        if s % 2 == 0:
            gens.append([(c.g_attn.copy(), c.g_ffn.copy()) for c in orc.caches])
        if s == 1:   # first interval: no previous generation -> plain reuse
            want = x + sum(g[0] + g[1] for g in gens[0])
            np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
        if s == 3:   # second interval: cur + (cur - prev) * 1/2 on every layer
            want = x.copy()
            for (ga0, gf0), (ga1, gf1) in zip(gens[0], gens[1]):
                want = want + (ga1 + (ga1 - ga0) * 0.5) + (gf1 + (gf1 - gf0) * 0.5)
            np.testing.assert_allclose(y, want, rtol=1e-12, atol=1e-12)
        x = euler_update(x, y, text0, cfg.n_text, 4)


def test_schedule_state_machine():
    cfg = get_config("tiny")
    ws, x0 = setup(cfg)
    orc = O.HeroOracle(cfg, ws)
    with pytest.raises(RuntimeError):
        orc.step(x0, 1)            # cached step before any full step
    orc2, outs = run_schedule(cfg, ws, x0, cfg.n_steps)
    assert orc2.n_full == 3 and orc2.last_full == 8      # full at 0, 4, 8 of 10 steps, M=4
    assert orc2.caches[1].g_attn_prev is not None        # deep layer kept two generations
    assert orc2.caches[0].g_attn_prev is None            # shallow layer does not
    assert orc2.caches[0].k is not None and orc2.caches[1].k is None
    assert all(np.isfinite(o).all() for o in outs)
    # step 9 is a cached step with k = 1 after the full step 8
    assert orc2.last_idx is not None and len(orc2.last_idx) == 64


def test_deep_cache_not_modified_on_cached_steps():
    cfg = get_config("tiny")
    ws, x0 = setup(cfg)
    orc = O.HeroOracle(cfg, ws)
    y = orc.step(x0, 0)
    snap = orc.caches[1].g_attn.copy(), orc.caches[1].g_ffn.copy()
    orc.step(y, 1)
    orc.step(y, 2)
    np.testing.assert_array_equal(orc.caches[1].g_attn, snap[0])
    np.testing.assert_array_equal(orc.caches[1].g_ffn, snap[1])


def test_in_place_cache_reading_for_m_greater_than_2():
    """A row refreshed at k=1 and not at k=2 reuses its k=1 value at k=2."""
    cfg = get_config("tiny", n_layers=1, n_shallow=1)
    ws, x0 = setup(cfg)
    orc = O.HeroOracle(cfg, ws)
    orc.full_layer(0, x0)
    x1 = perturb_tokens(x0.astype(np.float32), 7, 0.3).astype(np.float64)
    orc.refresh_layer(0, x1, np.array([50]))
    after_k1 = orc.caches[0].g_attn[50].copy()
    orc.refresh_layer(0, x1, np.array([51]))
    np.testing.assert_array_equal(orc.caches[0].g_attn[50], after_k1)


def test_token_order_is_immaterial():
    """Permuting the joint sequence permutes the outputs (attention has no positions)."""
    cfg = get_config("tiny", n_layers=1, n_shallow=1)
    ws, x0 = setup(cfg)
    w = O._cast_weights(ws[0], np.float64)
    perm = np.random.default_rng(9).permutation(cfg.n_tokens)
    y = O.block_forward(x0, w, cfg.n_heads, cfg.ln_eps)[0]
    yp = O.block_forward(x0[perm], w, cfg.n_heads, cfg.ln_eps)[0]
    np.testing.assert_allclose(yp, y[perm], rtol=1e-9, atol=1e-11)
