"""GPU parity at the full workload sizes (CogVideoX-2B / 5B shaped blocks, long video), in the
launch configuration bench.py times.

The float64 oracle cannot run a whole 17 776-token block in seconds, so after a full layer it
computes what is cheap in full (K and V of every row: one GEMM) and the features on sampled
rows; after a refresh it computes EVERY refreshed row (the rows the method recomputes), and
sampled non-refreshed and text rows.  Selection indices and ages are compared in full, bit for
bit.  One test runs hero_step itself, at a size where it takes its deferred-residual path,
against the oracle's step.
"""
import numpy as np
import pytest
import torch

from oracle import hero_oracle as O
from paper_2508_17588_amd import binding as B
from workloads import (RATIO_SWEEP, BLOCK_ADALN, BLOCK_QKNORM, BLOCK_ROPE, get_config, make_block_extras,
                       make_layer_weights, make_tokens, perturb_tokens)
from block_oracle import BlockOracle
from hero_testlib import assert_close, to_dev_bf16, to_host_f64, upload_weights

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", flush=True)


def rows_in_chunks(orc, x64, rows, k_all, v_all, chunk=2304):
    """orc.rows over many rows, a few thousand at a time (the score matrix of a chunk is chunk x N)."""
    parts = [orc.rows(x64[rows[i:i + chunk]], rows[i:i + chunk], k_all, v_all) for i in range(0, len(rows), chunk)]
    return tuple(np.concatenate([p[j] for p in parts]) for j in range(3))


def sample_rows(cfg, idx, rng, n_each=20):
    idx = np.asarray(idx, np.int64)
    sel = rng.choice(idx, size=min(n_each, len(idx)), replace=False)
    sel = np.unique(np.concatenate([sel, idx[:2], idx[-2:]]))          # first and last picks too
    others = np.setdiff1d(np.arange(cfg.n_text, cfg.n_tokens), idx)
    non = rng.choice(others, size=min(n_each, len(others)), replace=False) if len(others) else np.zeros(0, np.int64)
    text = np.array([0, cfg.n_text - 1], np.int64)
    return sel, np.unique(non), text


def run_block(base_name, sweeps, block_flags=0, every_row=("10", "25", "50", "paper"), via_step=False):
    """One block at full size: fill, select, refresh -- through the per-layer entry points, or with
    via_step through hero_step itself (steps 0 and 1 of a one-layer model with M = 2; at these sizes
    the cached step takes hero_step's deferred-residual path: refreshed rows of x updated by the
    FFN2 kernel, all other rows by the end-of-step pass).  K and V are compared on every element.  The
    features S and the increment of x are compared on sampled rows after the fill and, after the
    refresh, on EVERY refreshed row for the sweeps named in every_row (else on sampled rows),
    against the float64 oracle with the oracle's ideal bf16 pipeline (block_oracle, stored_bf16)
    as the second reference that hero_testlib.assert_close describes."""
    base = get_config(base_name).with_(n_layers=1, n_shallow=1, block_flags=block_flags)
    rng = np.random.default_rng(5)
    w = make_layer_weights(base, 0, seed=0)
    if block_flags:
        w.update(make_block_extras(base, 0, seed=0, step=0))
    orc, orc16 = BlockOracle(base, w), BlockOracle(base, w, stored_bf16=True)
    x0 = make_tokens(base, seed=1)
    x1 = perturb_tokens(x0, seed=2, std=0.1)
    x0_64, x1_64 = x0.astype(np.float64), x1.astype(np.float64)
    say(f"{base_name}: oracle K/V of all {base.n_tokens} rows (exact and ideal bf16 pipeline)")
    all_rows = np.arange(base.n_tokens)
    k0, v0 = orc.kv(x0_64, all_rows)
    k0_16, v0_16 = orc16.kv(x0_64, all_rows)

    for tag, over in sweeps:
        cfg = base.with_(**over)
        say(f"{base_name} [{tag}]: full layer on the GPU")
        cache = B.HeroCache(B.make_config(cfg))
        upload_weights(cache, cfg, [w])
        xd = torch.from_numpy(x0).cuda()
        if via_step:
            assert cfg.n_layers == 1 and cfg.interval == 2 and tag != "100"
            cache.hero_step(xd, 0)
        else:
            cache.hero_full_layer(0, xd)
        torch.cuda.synchronize()
        # --- the fill: K, V in full; S and x on sampled rows
        assert_close(to_host_f64(cache.hero_cache_view(0, B.VIEW_K)), k0, f"{base_name} {tag} fill: K", emul=k0_16)
        vt = to_host_f64(cache.hero_cache_view(0, B.VIEW_VT))
        assert_close(vt[:, :cfg.n_tokens].T, v0, f"{base_name} {tag} fill: V", emul=v0_16)
        assert float(np.abs(vt[:, cfg.n_tokens:]).max(initial=0.0)) == 0.0
        del vt
        probe = np.unique(np.concatenate([rng.choice(cfg.n_tokens, 24, replace=False), [0, cfg.n_tokens - 1]]))
        ga, gf, s_want = orc.rows(x0_64[probe], probe, k0, v0)
        _, _, s_ideal = orc16.rows(x0_64[probe], probe, k0_16, v0_16)
        s_gpu = cache.hero_cache_view(0, B.VIEW_S_CUR)
        # (the attention feature is stored in bf16 before the FFN feature is added to it)
        assert_close(to_host_f64(s_gpu[probe]), s_want, f"{base_name} {tag} fill: S rows", stored_parts=[ga], emul=s_ideal)
        # x is updated in fp32 by the stored (bf16) feature sum: judge the increment at its own scale
        assert_close(to_host_f64(xd[probe]) - x0_64[probe], s_want, f"{base_name} {tag} fill: x increment rows",
                     stored_parts=[ga], emul=s_ideal)

        # --- the cached step: select (bit-exact, in full), refresh
        if tag == "100":
            idx_np = np.arange(cfg.n_tokens, dtype=np.int32)            # all rows incl. text
            idx_d = torch.from_numpy(idx_np).cuda()
        elif not via_step:
            n_sel = B.hero_num_selected(cache.cfg)
            idx_d = torch.empty(n_sel, dtype=torch.int32, device="cuda")
            cache.hero_reset_ages()
            assert cache.hero_select(1, idx_d) == n_sel
            idx_np, ages = O.select(np.zeros(cfg.n_video, np.int32), cfg, 1)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(idx_d.cpu().numpy(), idx_np)
            np.testing.assert_array_equal(cache.hero_cache_view(0, B.VIEW_AGES).cpu().numpy(), ages)
        else:
            idx_np, ages = O.select(np.zeros(cfg.n_video, np.int32), cfg, 1)
        say(f"{base_name} [{tag}]: refresh of {len(idx_np)} rows")
        s_before = s_gpu.clone()
        xd = torch.from_numpy(x1).cuda()
        if via_step:
            cache.hero_profile_begin()
            cache.hero_step(xd, 1)
            prof = cache.hero_profile_end()
            # the deferred path: no residual pass per layer, one pass at the end of the step
            assert "resid/cached" not in prof and prof["extrap/cached"][1] == 1, sorted(prof)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(cache.hero_cache_view(0, B.VIEW_IDX).cpu().numpy(), idx_np)
            np.testing.assert_array_equal(cache.hero_cache_view(0, B.VIEW_AGES).cpu().numpy(), ages)
        else:
            cache.hero_refresh_layer(0, xd, idx_d, len(idx_np))
        torch.cuda.synchronize()
        rows64 = idx_np.astype(np.int64)
        k1, v1, k1_16, v1_16 = k0.copy(), v0.copy(), k0_16.copy(), v0_16.copy()
        k1[rows64], v1[rows64] = orc.kv(x1_64[rows64], rows64)
        k1_16[rows64], v1_16[rows64] = orc16.kv(x1_64[rows64], rows64)
        assert_close(to_host_f64(cache.hero_cache_view(0, B.VIEW_K)), k1, f"{base_name} {tag} refresh: K", emul=k1_16)
        assert_close(to_host_f64(cache.hero_cache_view(0, B.VIEW_VT))[:, :cfg.n_tokens].T, v1, f"{base_name} {tag} refresh: V",
                     emul=v1_16)
        if tag == "100":
            sel = np.unique(np.concatenate([rng.choice(cfg.n_tokens, 24, replace=False), [0, cfg.n_tokens - 1]]))
            non, text = np.zeros(0, np.int64), np.zeros(0, np.int64)
        else:
            sel, non, text = sample_rows(cfg, idx_np, rng)
            if tag in every_row:
                sel = np.sort(rows64)
            elif len(rows64) > 2000:
                sel = np.unique(np.concatenate([sel, rows64[::7]]))     # every 7th pick: some rows of every query block
        say(f"{base_name} [{tag}]: oracle on {len(sel)} of the {len(idx_np)} refreshed rows")
        ga, gf, s_want = rows_in_chunks(orc, x1_64, sel, k1, v1)
        _, _, s_ideal = rows_in_chunks(orc16, x1_64, sel, k1_16, v1_16)
        sel_d = torch.from_numpy(sel).cuda()
        assert_close(to_host_f64(s_gpu[sel_d]), s_want, f"{base_name} {tag} refresh: S of {len(sel)} refreshed rows",
                     stored_parts=[ga], emul=s_ideal)
        assert_close(to_host_f64(xd[sel_d]) - x1_64[sel], s_want, f"{base_name} {tag} refresh: x increment of {len(sel)} refreshed rows",
                     stored_parts=[ga], emul=s_ideal)
        keep = np.concatenate([non, text]).astype(np.int64)
        if len(keep):
            assert torch.equal(s_gpu[keep], s_before[keep])             # reused rows untouched
            want = x1_64[keep] + to_host_f64(s_before[keep])
            np.testing.assert_allclose(to_host_f64(xd[keep]), want, rtol=0, atol=2e-6)
            # and those reused features are the full step's: check against the oracle too
            ga0, gf0, s0_want = orc.rows(x0_64[keep], keep, k0, v0)
            _, _, s0_ideal = orc16.rows(x0_64[keep], keep, k0_16, v0_16)
            assert_close(to_host_f64(xd[keep]) - x1_64[keep], s0_want, f"{base_name} {tag} refresh: x increment of reused rows",
                         stored_parts=[ga0], emul=s0_ideal)
        cache.close()
        del cache, s_gpu, s_before, xd
        torch.cuda.empty_cache()


def test_cvx2b_block_quarter_refresh():
    """Config 2: one CogVideoX-2B-shaped block, 17 776 tokens, 25 % patch-wise refresh, run through
    hero_step (a full step, then a cached step that takes the deferred-residual path); every
    refreshed row against the oracle."""
    run_block("cvx2b_block", [("25", {})], via_step=True)


def test_cvx5b_block_ratio_sweep():
    """Config 3: one CogVideoX-5B-shaped block, refresh ratio 10 / 25 / 50 / 100 %; every refreshed
    row of the 10, 25 and 50 % refreshes is compared with the oracle."""
    run_block("cvx5b_block", [("10", RATIO_SWEEP["10"]), ("25", RATIO_SWEEP["25"]),
                              ("50", RATIO_SWEEP["50"]), ("100", {})])


def test_cvx5b_block_paper_geometry():
    """The paper's operating geometry (Sec. 4.1: 2 x 3 patches, R = 0.2 -> one token of six, 2925
    refreshed rows) on one 5B-shaped block, run through hero_step (a full step, then a cached step
    that takes the deferred-residual path); every refreshed row against the oracle."""
    run_block("cvx5b_block", [("paper", dict(patch_h=2, patch_w=3, ratio=0.2))], via_step=True)


def test_cvx5b_block_modulated():
    """Config 3's block with adaLN modulation, q/k LayerNorm and rotary positions, 25 % refresh,
    every refreshed row.  The gates and (1 + scale) factors (1 + N(0, 0.1) per channel) multiply the
    branch features and with them the absolute error of any bf16 pipeline; the same criterion as for
    the plain block applies (flat 2e-2, or within an ulp of the oracle's ideal bf16 pipeline)."""
    run_block("cvx5b_block", [("25", RATIO_SWEEP["25"])], block_flags=BLOCK_ADALN | BLOCK_QKNORM | BLOCK_ROPE)


def test_cvx5b_long_video_refresh_and_extrapolation():
    """Config 5: 33 976 tokens; refresh at 25 %, and deep-layer extrapolation over the
    [33976, 3072] bf16 feature cache checked on every element."""
    run_block("cvx5b_long", [("25", {})], every_row=())
    cfg = get_config("cvx5b_long")                       # layer 0 shallow, layer 1 deep
    say("cvx5b_long: two full steps of the deep layer, then extrapolation k=1 of M=2")
    cache = B.HeroCache(B.make_config(cfg))
    w = [make_layer_weights(cfg, l, seed=0) for l in range(2)]
    upload_weights(cache, cfg, w)
    x0 = make_tokens(cfg, seed=1)
    for seed in (0, 3):
        xd = torch.from_numpy(x0 if seed == 0 else perturb_tokens(x0, seed=seed, std=0.1)).cuda()
        cache.hero_full_layer(1, xd)
    torch.cuda.synchronize()
    s_cur = to_host_f64(cache.hero_cache_view(1, B.VIEW_S_CUR))
    s_prev = to_host_f64(cache.hero_cache_view(1, B.VIEW_S_PREV))
    assert np.abs(s_cur - s_prev).max() > 0
    # the cached generations themselves: sampled rows against the oracle
    orc = BlockOracle(cfg, w[1])
    x3 = perturb_tokens(x0, seed=3, std=0.1).astype(np.float64)
    k3, v3 = orc.kv(x3, np.arange(cfg.n_tokens))
    probe = np.array([0, 225, 226, 5000, 20000, cfg.n_tokens - 1])
    ga, gf, s_want = orc.rows(x3[probe], probe, k3, v3)
    assert_close(s_cur[probe], s_want, "deep layer: S_cur rows", stored_parts=[ga])
    x2 = perturb_tokens(x0, seed=4, std=0.1)
    xd = torch.from_numpy(x2).cuda()
    cache.hero_extrapolate_layer(1, xd, 1)
    torch.cuda.synchronize()
    want = x2.astype(np.float64) + s_cur + (s_cur - s_prev) * 0.5      # Eq. 5 with k/M = 1/2
    np.testing.assert_allclose(to_host_f64(xd), want, rtol=0, atol=4e-6)
    cache.close()


@pytest.mark.parametrize("resid_fp32", [True, False])
def test_hero_step_with_deferred_residual_adds_against_the_oracle_step(resid_fp32):
    """hero_step on a problem large enough for its deferred-residual path (the FFN2 problem of a
    cached step has 9 x 16 = 144 tiles of 256 x 256, so the FFN2 kernel updates the refreshed rows
    of x and one pass at the end of the step adds the cached features of all other rows and the
    deep stack), against Alg. 1 as the oracle runs it, layer by layer with a residual add per
    layer: four steps (full, cached, full, cached; M = 2), two shallow and two deep layers, hidden
    4096 (64 heads), 2848 tokens of which 2112 are refreshed (1 x 4 patches, three of four tokens).
    Wide and short, because the oracle's cost is in its per-head score matrices.  The oracle runs
    in float32 here (its plain definitions at single precision: that error, ~1e-6 relative, is far
    below the bf16 tolerance), which halves its time to about a minute.
    With a bf16 residual stream (two steps only) x is rounded to bf16 by every kernel that updates it
    -- the FFN2 kernel per layer on the rows it owns, the end-of-step pass once on all others -- so the
    bound of its increment grows by one half-ulp of x per layer."""
    cfg = get_config("cvx5b_42l").with_(n_layers=4, n_shallow=2, interval=2, hidden=4096, n_heads=64, head_dim=64,
                                        ffn_dim=1024, frames=1, height=44, width=64, n_text=32, patch_h=1, patch_w=4,
                                        ratio=0.75)
    ws = [make_layer_weights(cfg, l, seed=0, std=0.015, ln_affine_noise=0.1) for l in range(cfg.n_layers)]
    cache = B.HeroCache(B.make_config(cfg, resid_fp32=resid_fp32))
    upload_weights(cache, cfg, ws)
    n_sel = B.hero_num_selected(cache.cfg)
    assert n_sel == 2112 and (n_sel + 255) // 256 * (cfg.hidden // 256) >= 128      # the size that defers
    orc = O.HeroOracle(cfg, ws, dtype=np.float32)
    x0 = make_tokens(cfg, seed=1)
    for step in range(4 if resid_fp32 else 2):
        say(f"deferred-residual hero_step vs oracle: step {step} (residual stream {'fp32' if resid_fp32 else 'bf16'})")
        x_in = x0 if step == 0 else perturb_tokens(x0, seed=30 + step, std=0.1)
        xd = torch.from_numpy(x_in).cuda()
        if not resid_fp32:
            xd = xd.to(torch.bfloat16)
        cache.hero_profile_begin()
        cache.hero_step(xd, step)
        prof = cache.hero_profile_end()
        if step % 2:
            # the deferred path: no per-layer residual pass, one pass at the end of the step
            assert "resid/cached" not in prof and prof["extrap/cached"][1] == 1, sorted(prof)
        want = orc.step(x_in, step).astype(np.float64)
        torch.cuda.synchronize()
        x64 = x_in.astype(np.float64)
        # The increment of x over the step is a sum of stored features, each inside the per-call
        # tolerance with an error of its own: one per layer on a full step and per shallow layer of a
        # cached step, and (1 + k/M) S_t - (k/M) S_{t+M} per deep layer (Eq. 5), whose two terms carry
        # their errors times 1.5 and 0.5 here.  Independent errors add in quadrature.
        alpha = 0.5 if step == 3 else 0.0
        coeff2 = 4.0 if step % 2 == 0 else 2.0 + 2.0 * ((1.0 + alpha) ** 2 + alpha ** 2)
        if resid_fp32:
            assert_close(to_host_f64(xd) - x64, want - x64, f"deferred step {step}: x increment over four layers",
                         max_abs=2e-2 * np.sqrt(coeff2))
        else:
            # a bf16 stream is judged as a stream: x itself, rounded once per layer on the way
            assert_close(to_host_f64(xd), want, f"deferred step {step}: x (bf16 stream) after four layers",
                         max_abs=2e-2 * np.sqrt(coeff2), stored_parts=[want] * (cfg.n_layers - 1))
        if step % 2:
            np.testing.assert_array_equal(cache.hero_cache_view(0, B.VIEW_IDX).cpu().numpy(), orc.last_idx)
        np.testing.assert_array_equal(cache.hero_cache_view(0, B.VIEW_AGES).cpu().numpy(), orc.ages)
        for l in range(cfg.n_layers):
            c = orc.caches[l]
            assert_close(to_host_f64(cache.hero_cache_view(l, B.VIEW_S_CUR)), c.g_attn.astype(np.float64) + c.g_ffn,
                         f"deferred step {step}: S of layer {l}", stored_parts=[c.g_attn])
            if l < cfg.n_shallow:
                assert_close(to_host_f64(cache.hero_cache_view(l, B.VIEW_K)), c.k, f"deferred step {step}: K of layer {l}")
                vt = to_host_f64(cache.hero_cache_view(l, B.VIEW_VT))
                assert_close(vt[:, :cfg.n_tokens].T, c.v, f"deferred step {step}: V of layer {l}")
            elif c.g_attn_prev is not None:
                assert_close(to_host_f64(cache.hero_cache_view(l, B.VIEW_S_PREV)),
                             c.g_attn_prev.astype(np.float64) + c.g_ffn_prev, f"deferred step {step}: S_prev of layer {l}")
    cache.close()


@pytest.mark.parametrize("n_layers,n_shallow", [(4, 2), (3, 2), (2, 2)])
def test_cached_step_with_deferred_residual_adds_matches_the_per_layer_calls(n_layers, n_shallow):
    """At this size hero_step defers the residual adds of a cached step: refreshed rows are updated
    by the FFN2 kernel layer by layer, all other rows once at the end of the step together with the
    deep stack.  It must agree, up to the order of fp32 additions, with the per-layer entry points
    (each of which is checked against the oracle elsewhere), and leave the same caches."""
    cfg = get_config("cvx5b_42l").with_(n_layers=n_layers, n_shallow=n_shallow, interval=2)
    say(f"cvx5b shape, {n_layers} layers ({n_shallow} shallow): hero_step vs per-layer calls over 4 steps")
    ws = [make_layer_weights(cfg, l, seed=0) for l in range(n_layers)]
    a, b = B.HeroCache(B.make_config(cfg)), B.HeroCache(B.make_config(cfg))
    upload_weights(a, cfg, ws)
    upload_weights(b, cfg, ws)
    n_sel = B.hero_num_selected(a.cfg)
    idx = torch.empty(n_sel, dtype=torch.int32, device="cuda")
    x0 = make_tokens(cfg, seed=1)
    for step in range(4):
        xin = torch.from_numpy(x0 if step == 0 else perturb_tokens(x0, seed=10 + step, std=0.1)).cuda()
        xa, xb = xin.clone(), xin.clone()
        a.hero_step(xa, step)
        if step % 2 == 0:
            for l in range(n_layers):
                b.hero_full_layer(l, xb)
            b.hero_reset_ages()
        else:
            assert b.hero_select(step, idx) == n_sel
            for l in range(n_shallow):
                b.hero_refresh_layer(l, xb, idx, n_sel)
            for l in range(n_shallow, n_layers):
                b.hero_extrapolate_layer(l, xb, 1)
        torch.cuda.synchronize()
        diff = float((xa - xb).abs().max())
        assert diff <= 5e-5, f"step {step}: x differs by {diff:.3e}"
        assert torch.equal(a.hero_cache_view(0, B.VIEW_AGES), b.hero_cache_view(0, B.VIEW_AGES))
        for l in range(n_layers):
            assert torch.equal(a.hero_cache_view(l, B.VIEW_S_CUR), b.hero_cache_view(l, B.VIEW_S_CUR)), (step, l)
    a.close()
    b.close()


def test_the_42_layer_workload_step_matches_the_per_layer_calls():
    """Config 4 as bench.py runs it (42 layers, 8 shallow, full step every 4th, 17 776 tokens):
    six steps of hero_step against the per-layer entry points, each of which is checked against the
    oracle at this shape above.  One set of weights serves every layer (the kernels and the schedule
    do not care, and 42 sets would be 9.5 GB of host draws).  Selection against the oracle, caches
    bit for bit, x up to the order of its fp32 additions (84 per row and step)."""
    cfg = get_config("cvx5b_42l")
    say("cvx5b_42l: hero_step vs per-layer calls over 6 steps (full at 0 and 4)")
    w = make_layer_weights(cfg, 0, seed=0)
    dev = {n: to_dev_bf16(w[n]) for n in w}
    a, b = B.HeroCache(B.make_config(cfg)), B.HeroCache(B.make_config(cfg))
    for l in range(cfg.n_layers):
        a.hero_set_layer_weights(l, dev)
        b.hero_set_layer_weights(l, dev)
    n_sel = B.hero_num_selected(a.cfg)
    idx = torch.empty(n_sel, dtype=torch.int32, device="cuda")
    ages = np.zeros(cfg.n_video, np.int32)
    x0 = make_tokens(cfg, seed=1)
    last_full = 0
    for step in range(6):
        say(f"  step {step}")
        xin = torch.from_numpy(x0 if step == 0 else perturb_tokens(x0, seed=20 + step, std=0.1)).cuda()
        xa, xb = xin.clone(), xin.clone()
        a.hero_step(xa, step)
        if step % cfg.interval == 0:
            last_full = step
            for l in range(cfg.n_layers):
                b.hero_full_layer(l, xb)
            b.hero_reset_ages()
            ages[:] = 0
        else:
            assert b.hero_select(step, idx) == n_sel
            want_idx, ages = O.select(ages, cfg, step)
            np.testing.assert_array_equal(idx.cpu().numpy(), want_idx)
            np.testing.assert_array_equal(a.hero_cache_view(0, B.VIEW_IDX).cpu().numpy(), want_idx)
            for l in range(cfg.n_shallow):
                b.hero_refresh_layer(l, xb, idx, n_sel)
            for l in range(cfg.n_shallow, cfg.n_layers):
                b.hero_extrapolate_layer(l, xb, step - last_full)
        torch.cuda.synchronize()
        assert torch.isfinite(xa).all()
        scale = float(xb.abs().max())
        diff = float((xa - xb).abs().max())
        assert diff <= 1e-5 * scale + 5e-5, f"step {step}: x differs by {diff:.3e} at |x| up to {scale:.1f}"
        np.testing.assert_array_equal(a.hero_cache_view(0, B.VIEW_AGES).cpu().numpy(), ages)
        assert torch.equal(a.hero_cache_view(0, B.VIEW_AGES), b.hero_cache_view(0, B.VIEW_AGES))
        for l in range(cfg.n_layers):
            assert torch.equal(a.hero_cache_view(l, B.VIEW_S_CUR), b.hero_cache_view(l, B.VIEW_S_CUR)), (step, l)
    a.close()
    b.close()
