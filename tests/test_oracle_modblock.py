"""Pins for the oracle's modulated block (adaLN shift/scale/gate, per-head q/k LayerNorm,
3-D rotary positions).  The paper leaves these internals out (Sec. 3.2, "omitting scale and
shift for clarity"), so each piece is pinned against its textbook definition: library routines,
rotation invariants, hand-computed angles, and reductions to the plain block."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import hero_oracle as O
from workloads import (BLOCK_ADALN, BLOCK_QKNORM, BLOCK_ROPE, MOD_ROWS, get_config, make_block_extras,
                       make_layer_weights, make_tokens, perturb_tokens)

ALL = BLOCK_ADALN | BLOCK_QKNORM | BLOCK_ROPE


def weights(cfg, layer=0, std=0.05, step=0):
    w = make_layer_weights(cfg, layer, seed=0, std=std, ln_affine_noise=0.1)
    w.update(make_block_extras(cfg, layer, seed=0, step=step))
    return {k: v.astype(np.float64) for k, v in w.items()}


def test_flag_and_row_order_constants_agree_with_the_input_generator():
    assert (O.BLOCK_ADALN, O.BLOCK_QKNORM, O.BLOCK_ROPE) == (BLOCK_ADALN, BLOCK_QKNORM, BLOCK_ROPE)
    assert O.MOD_ROWS == MOD_ROWS


def test_stream_vector_picks_text_and_video_rows():
    mod = np.arange(12 * 4, dtype=np.float64).reshape(12, 4)
    got = O.stream_vector(mod, "gate2", np.array([0, 2, 3, 7]), n_text=3)
    np.testing.assert_array_equal(got[0], mod[MOD_ROWS.index("gate2_t")])
    np.testing.assert_array_equal(got[1], mod[MOD_ROWS.index("gate2_t")])
    np.testing.assert_array_equal(got[2], mod[MOD_ROWS.index("gate2_v")])
    np.testing.assert_array_equal(got[3], mod[MOD_ROWS.index("gate2_v")])


def test_head_layer_norm_is_the_library_layer_norm_per_head():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 4 * 32)) * 3 + 1
    g, b = rng.standard_normal(32), rng.standard_normal(32)
    want = F.layer_norm(torch.from_numpy(x).reshape(7, 4, 32), (32,), torch.from_numpy(g), torch.from_numpy(b), 1e-6)
    np.testing.assert_allclose(O.head_layer_norm(x, g, b, 4), want.reshape(7, 128).numpy(), rtol=1e-12, atol=1e-12)


def test_modulated_layer_norm_against_the_library():
    cfg = get_config("tiny", block_flags=BLOCK_ADALN)
    w = weights(cfg)
    ext = O.BlockExt(cfg)
    x = make_tokens(cfg, seed=1).astype(np.float64)
    rows = np.array([0, cfg.n_text - 1, cfg.n_text, cfg.n_tokens - 1])
    for which in (1, 2):
        base = F.layer_norm(torch.from_numpy(x[rows]), (cfg.hidden,), torch.from_numpy(w[f"ln{which}_g"]),
                            torch.from_numpy(w[f"ln{which}_b"]), cfg.ln_eps).numpy()
        for i, r in enumerate(rows):
            s = "t" if r < cfg.n_text else "v"
            want = base[i] * (1 + w["mod"][MOD_ROWS.index(f"scale{which}_{s}")]) + w["mod"][MOD_ROWS.index(f"shift{which}_{s}")]
            np.testing.assert_allclose(ext.ln(x[rows], rows, w, which, cfg.ln_eps)[i], want, rtol=1e-12, atol=1e-12)


def test_rope_angles_hand_computed():
    # head_dim 16: 2 pairs for t, 3 for y, 3 for x; token (t=1, y=2, x=3) of a 2 x 3 x 4 grid
    ang = O.rope_angles(2, 3, 4, 16)
    assert ang.shape == (24, 8)
    th = 10000.0
    tok = (1 * 3 + 2) * 4 + 3
    want = [1 * 1.0, 1 * th ** -0.5, 2 * 1.0, 2 * th ** (-1 / 3), 2 * th ** (-2 / 3), 3 * 1.0, 3 * th ** (-1 / 3), 3 * th ** (-2 / 3)]
    np.testing.assert_allclose(ang[tok], want, rtol=1e-14)
    np.testing.assert_array_equal(ang[0], np.zeros(8))                 # the origin is not rotated
    # head_dim 64 splits 8 / 12 / 12 pairs = 16 / 24 / 24 channels
    a64 = O.rope_angles(1, 1, 2, 64)
    assert a64.shape == (2, 32) and (a64[1, :20] == 0).all() and (a64[1, 20:] > 0).all()


def test_rope_is_a_rotation_and_depends_on_relative_position_only():
    rng = np.random.default_rng(1)
    heads, hd = 2, 64
    ang = O.rope_angles(3, 4, 5, hd)
    q = rng.standard_normal((60, heads * hd))
    k = rng.standard_normal((60, heads * hd))
    rq, rk = O.apply_rope(q, ang, heads), O.apply_rope(k, ang, heads)
    # pairwise norms are kept
    np.testing.assert_allclose((rq.reshape(60, -1, 2) ** 2).sum(-1), (q.reshape(60, -1, 2) ** 2).sum(-1), rtol=1e-12)
    # complex form: (a + ib) e^{i phi}
    z = (q.reshape(60, heads, hd // 2, 2)[..., 0] + 1j * q.reshape(60, heads, hd // 2, 2)[..., 1]) * np.exp(1j * ang)[:, None, :]
    np.testing.assert_allclose(rq.reshape(60, heads, hd // 2, 2)[..., 0], z.real, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(rq.reshape(60, heads, hd // 2, 2)[..., 1], z.imag, rtol=1e-12, atol=1e-12)
    # the score of one (q, k) content pair placed at positions p and p' depends on p - p' only
    def tok(t, y, x): return (t * 4 + y) * 5 + x
    q0, k0 = q[:1], k[:1]
    def score(pq, pk):
        a = O.apply_rope(q0, ang[[tok(*pq)]], heads)
        b = O.apply_rope(k0, ang[[tok(*pk)]], heads)
        return (a.reshape(heads, hd) * b.reshape(heads, hd)).sum(-1)
    np.testing.assert_allclose(score((0, 1, 1), (1, 3, 2)), score((1, 1, 3), (2, 3, 4)), rtol=1e-10)
    np.testing.assert_allclose(score((2, 0, 4), (0, 2, 1)), score((2, 1, 4), (0, 3, 1)), rtol=1e-10)
    assert not np.allclose(score((0, 1, 1), (1, 3, 2)), score((0, 1, 1), (1, 3, 3)))


def run_full(cfg, w, x):
    orc = O.HeroOracle(cfg, [w])
    y = orc.full_layer(0, x)
    return y, orc


def test_identity_modulation_reduces_to_the_plain_block():
    cfg0 = get_config("tiny", n_layers=1, n_shallow=1)
    cfg1 = cfg0.with_(block_flags=BLOCK_ADALN)
    w = weights(cfg0)
    for i, nm in enumerate(MOD_ROWS):
        w["mod"][i] = 1.0 if nm.startswith("gate") else 0.0
    x = make_tokens(cfg0, seed=1).astype(np.float64)
    y0, o0 = run_full(cfg0, w, x)
    y1, o1 = run_full(cfg1, w, x)
    np.testing.assert_allclose(y1, y0, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(o1.caches[0].g_ffn, o0.caches[0].g_ffn, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(o1.caches[0].k, o0.caches[0].k, rtol=1e-12, atol=1e-12)


def test_gates_scale_the_cached_features_per_stream():
    cfg = get_config("tiny", n_layers=1, n_shallow=1, block_flags=BLOCK_ADALN)
    w = weights(cfg)
    x = make_tokens(cfg, seed=1).astype(np.float64)
    _, o = run_full(cfg, w, x)
    w2 = {k: v.copy() for k, v in w.items()}
    w2["mod"][MOD_ROWS.index("gate1_v")] *= 2.0             # doubles the attention feature of video rows only
    w2["mod"][MOD_ROWS.index("gate2_t")] = 0.0              # removes the FFN feature of text rows
    _, o2 = run_full(cfg, w2, x)
    nt = cfg.n_text
    np.testing.assert_allclose(o2.caches[0].g_attn[nt:], 2.0 * o.caches[0].g_attn[nt:], rtol=1e-12)
    np.testing.assert_allclose(o2.caches[0].g_attn[:nt], o.caches[0].g_attn[:nt], rtol=1e-12)
    assert (o2.caches[0].g_ffn[:nt] == 0).all()
    # all gates zero: the block adds nothing
    w3 = {k: v.copy() for k, v in w.items()}
    for i, nm in enumerate(MOD_ROWS):
        if nm.startswith("gate"):
            w3["mod"][i] = 0.0
    y3, _ = run_full(cfg, w3, x)
    np.testing.assert_array_equal(y3, x)


def test_scale_minus_one_makes_the_branch_input_the_shift():
    """scale = -1 wipes the normalised input: attention then sees the same row everywhere
    (within a stream), so with one stream's shift equal to the other's every query gets the same
    value vector and the attention feature is the same on all rows."""
    cfg = get_config("tiny", n_layers=1, n_shallow=1, block_flags=BLOCK_ADALN)
    w = weights(cfg)
    for s in ("v", "t"):
        w["mod"][MOD_ROWS.index(f"scale1_{s}")] = -1.0
        w["mod"][MOD_ROWS.index(f"shift1_{s}")] = w["mod"][MOD_ROWS.index("shift1_v")]
        w["mod"][MOD_ROWS.index(f"gate1_{s}")] = 1.0
    x = make_tokens(cfg, seed=1).astype(np.float64)
    _, o = run_full(cfg, w, x)
    g = o.caches[0].g_attn
    np.testing.assert_allclose(g, np.broadcast_to(g[0], g.shape), rtol=1e-10, atol=1e-12)
    u = w["mod"][MOD_ROWS.index("shift1_v")]
    v_row = O.linear(u[None], w["w_qkv"], w["b_qkv"])[:, 2 * cfg.hidden:]
    np.testing.assert_allclose(g[0], O.linear(v_row, w["w_o"], w["b_o"])[0], rtol=1e-10, atol=1e-12)


def test_text_rows_are_not_rotated_and_video_rows_are():
    cfg = get_config("tiny", n_layers=1, n_shallow=1, block_flags=BLOCK_ROPE)
    cfg0 = cfg.with_(block_flags=0)
    w = weights(cfg)
    x = make_tokens(cfg, seed=1).astype(np.float64)
    _, o = run_full(cfg, w, x)
    _, o0 = run_full(cfg0, w, x)
    nt = cfg.n_text
    np.testing.assert_array_equal(o.caches[0].k[:nt], o0.caches[0].k[:nt])
    np.testing.assert_array_equal(o.caches[0].k[nt], o0.caches[0].k[nt])       # token (0,0,0): angle 0
    assert not np.allclose(o.caches[0].k[nt + 1:], o0.caches[0].k[nt + 1:])
    np.testing.assert_array_equal(o.caches[0].v, o0.caches[0].v)               # V is never rotated
    want = O.apply_rope(o0.caches[0].k[nt:], O.rope_angles(cfg.frames, cfg.height, cfg.width, cfg.head_dim), cfg.n_heads)
    np.testing.assert_allclose(o.caches[0].k[nt:], want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("flags", [BLOCK_ADALN, BLOCK_QKNORM, BLOCK_ROPE, ALL])
def test_refresh_of_all_rows_is_the_full_layer_and_refresh_is_local(flags):
    cfg = get_config("tiny", n_layers=1, n_shallow=1, block_flags=flags)
    w = weights(cfg)
    x0 = make_tokens(cfg, seed=1).astype(np.float64)
    x1 = perturb_tokens(make_tokens(cfg, seed=1), seed=2, std=0.1).astype(np.float64)
    orc = O.HeroOracle(cfg, [w])
    orc.full_layer(0, x0)
    before = {k: getattr(orc.caches[0], k).copy() for k in ("k", "v", "g_attn", "g_ffn")}
    # refresh of a few rows: others bit-unchanged
    idx = np.array([cfg.n_text + 3, cfg.n_text + 40, cfg.n_tokens - 1])
    y = orc.refresh_layer(0, x1, idx)
    keep = np.setdiff1d(np.arange(cfg.n_tokens), idx)
    for k_, v_ in before.items():
        np.testing.assert_array_equal(getattr(orc.caches[0], k_)[keep], v_[keep])
        assert not np.array_equal(getattr(orc.caches[0], k_)[idx], v_[idx])
    np.testing.assert_allclose(y, x1 + orc.caches[0].g_attn + orc.caches[0].g_ffn, rtol=1e-14)
    # refresh of every row == full layer on the new input
    y_all = orc.refresh_layer(0, x1, np.arange(cfg.n_tokens))
    ref = O.HeroOracle(cfg, [w])
    y_full = ref.full_layer(0, x1)
    np.testing.assert_allclose(y_all, y_full, rtol=1e-12, atol=1e-12)


def test_qk_norm_changes_scores_as_the_library_sdpa_sees_them():
    """Whole attention branch with q/k LayerNorm against torch: F.layer_norm per head, then
    F.scaled_dot_product_attention."""
    cfg = get_config("tiny", n_layers=1, n_shallow=1, block_flags=BLOCK_QKNORM)
    w = weights(cfg)
    x = make_tokens(cfg, seed=1).astype(np.float64)
    _, o = run_full(cfg, w, x)
    d, h, hd = cfg.hidden, cfg.n_heads, cfg.head_dim
    tw = {k: torch.from_numpy(v) for k, v in w.items()}
    u = F.layer_norm(torch.from_numpy(x), (d,), tw["ln1_g"], tw["ln1_b"], cfg.ln_eps)
    qkv = F.linear(u, tw["w_qkv"], tw["b_qkv"])
    q = F.layer_norm(qkv[:, :d].reshape(-1, h, hd), (hd,), tw["qn_g"], tw["qn_b"], 1e-6)
    k = F.layer_norm(qkv[:, d:2 * d].reshape(-1, h, hd), (hd,), tw["kn_g"], tw["kn_b"], 1e-6)
    v = qkv[:, 2 * d:].reshape(-1, h, hd)
    att = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1)).transpose(0, 1)
    g = F.linear(att.reshape(-1, d), tw["w_o"], tw["b_o"]).numpy()
    np.testing.assert_allclose(o.caches[0].g_attn, g, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(o.caches[0].k, k.reshape(-1, d).numpy(), rtol=1e-10, atol=1e-12)
