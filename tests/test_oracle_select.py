"""Pins for the oracle's selection function (Eq. 4 + frequency-aware tracking) and
the cost model read off the paper's Tables 3 and 4 (CPU only)."""
import math
import os

import numpy as np
import pytest

from oracle import hero_oracle as O
from workloads import get_config, RATIO_SWEEP

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def load_table(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append(line.split())
    return rows


# ---------------------------------------------------------------- hash

def _inv_xorshift(h, s):
    out = h
    for _ in range(32 // s + 1):
        out = h ^ (out >> s)
    return out


def _inv_fmix32(h):
    h = _inv_xorshift(h, 16)
    h = (h * pow(0xC2B2AE35, -1, 1 << 32)) & 0xFFFFFFFF
    h = _inv_xorshift(h, 13)
    h = (h * pow(0x85EBCA6B, -1, 1 << 32)) & 0xFFFFFFFF
    h = _inv_xorshift(h, 16)
    return h


def test_fmix32_is_the_stated_bijection():
    xs = np.random.default_rng(0).integers(0, 1 << 32, 2000, dtype=np.uint64)
    hs = O.fmix32(xs)
    assert hs.max() < (1 << 32)
    for x, h in zip(xs.tolist(), hs.tolist()):
        assert _inv_fmix32(h) == x      # inverse built from modular inverses, not from fmix32
    assert int(O.fmix32(np.uint64(0))) == 0
    # plain-python restatement on a few values
    def py(h):
        h ^= h >> 16; h = (h * 0x85EBCA6B) & 0xFFFFFFFF
        h ^= h >> 13; h = (h * 0xC2B2AE35) & 0xFFFFFFFF
        h ^= h >> 16
        return h
    for x in (1, 2, 0xDEADBEEF, 0xFFFFFFFF):
        assert int(O.fmix32(np.uint64(x))) == py(x)


def test_mix32_distinct_per_token_and_depends_on_step_and_seed():
    toks = np.arange(20000)
    h = O.mix32(1234, 3, toks)
    assert len(np.unique(h)) == len(toks)
    assert not np.array_equal(h, O.mix32(1234, 4, toks))
    assert not np.array_equal(h, O.mix32(1235, 3, toks))
    # avalanche: low bits are balanced
    assert abs((h & np.uint64(1)).mean() - 0.5) < 0.02
    assert abs(((h >> np.uint64(31)) & np.uint64(1)).mean() - 0.5) < 0.02


# ---------------------------------------------------------------- tokens per patch

def test_tokens_per_patch_rounding_matches_table3_spacing():
    """Table 3: R = .8 .7 .5 .3 .2 with 2x3 patches are equally spaced in FLOPs,
    which holds for 5,4,3,2,1 tokens per patch (round to nearest), not for floor or ceil."""
    rows = load_table("paper_table3_ratio_sweep.txt")
    ratios = [float(r[0]) for r in rows]
    flops = [float(r[2]) for r in rows]
    n = [O.tokens_per_patch(r, 6) for r in ratios]
    assert n == [5, 4, 3, 2, 1]
    gaps = [(flops[i] - flops[i + 1]) / (n[i] - n[i + 1]) for i in range(4)]
    assert max(gaps) - min(gaps) < 0.5          # 412.6 .. 412.9 T per token-per-patch
    assert [math.floor(r * 6) for r in ratios] != n and [math.ceil(r * 6) for r in ratios] != n


def test_tokens_per_patch_edges():
    assert O.tokens_per_patch(0.25, 4) == 1
    assert O.tokens_per_patch(0.25, 2) == 1      # clipped 2x1 edge patch: 0.5+0.5 -> 1
    assert O.tokens_per_patch(0.25, 6) == 2      # 1.5 + 0.5 -> 2 (half up)
    assert O.tokens_per_patch(0.10, 10) == 1
    assert O.tokens_per_patch(0.5, 4) == 2
    assert O.tokens_per_patch(1.0, 4) == 4
    assert O.tokens_per_patch(0.01, 4) == 1      # at least one
    assert O.tokens_per_patch(0.0, 4) == 0
    assert O.tokens_per_patch(2.0, 4) == 4       # clamped


def test_realised_refresh_counts_of_the_workloads():
    def count(cfg):
        return sum(O.tokens_per_patch(cfg.ratio, hh * ww) for (_, _, _, hh, ww) in
                   O.patch_list(cfg.frames, cfg.height, cfg.width, cfg.patch_h, cfg.patch_w))
    assert count(get_config("tiny")) == 64
    assert count(get_config("cvx5b_block")) == 4485
    assert count(get_config("cvx5b_block", **RATIO_SWEEP["10"])) == 1755
    assert count(get_config("cvx5b_block", **RATIO_SWEEP["50"])) == 8775
    assert count(get_config("cvx5b_long")) == 8625
    assert count(get_config("paper_point")) == 2925


# ---------------------------------------------------------------- selection invariants

@pytest.mark.parametrize("name,over", [
    ("tiny", {}),
    ("tiny", dict(height=7, width=9, patch_h=2, patch_w=3, ratio=0.34)),
    ("tiny", dict(frames=2, height=5, width=5, patch_h=3, patch_w=2, ratio=0.5)),
    ("reduced_42l", {}),
])
def test_selection_invariants(name, over):
    cfg = get_config(name, **over)
    patches = O.patch_list(cfg.frames, cfg.height, cfg.width, cfg.patch_h, cfg.patch_w)
    # patches partition the grid
    cover = np.zeros(cfg.n_video, int)
    for (t, y0, x0, hh, ww) in patches:
        for dy in range(hh):
            for dx in range(ww):
                cover[(t * cfg.height + y0 + dy) * cfg.width + x0 + dx] += 1
    assert (cover == 1).all()
    assert len(patches) == cfg.frames * math.ceil(cfg.height / cfg.patch_h) * math.ceil(cfg.width / cfg.patch_w)

    ages = np.zeros(cfg.n_video, np.int32)
    last_seen = np.zeros(cfg.n_video, int)
    worst_wait = max(math.ceil(hh * ww / O.tokens_per_patch(cfg.ratio, hh * ww)) for (_, _, _, hh, ww) in patches)
    for step in range(1, 4 * worst_wait + 1):
        idx, new_ages = O.select(ages, cfg, step)
        tok = idx.astype(int) - cfg.n_text
        assert idx.dtype == np.int32
        assert len(np.unique(idx)) == len(idx)                       # unique
        assert tok.min() >= 0 and tok.max() < cfg.n_video            # video rows only
        pos = 0
        for (t, y0, x0, hh, ww) in patches:                          # exactly n_p per patch, patch-major
            n_p = O.tokens_per_patch(cfg.ratio, hh * ww)
            for tk in tok[pos:pos + n_p]:
                tt, rem = divmod(tk, cfg.height * cfg.width)
                yy, xx = divmod(rem, cfg.width)
                assert tt == t and y0 <= yy < y0 + hh and x0 <= xx < x0 + ww
            # rank-minor: keys decrease inside the patch
            keys = [(int(ages[tk]) << 32) | int(O.mix32(cfg.seed, step, np.array([tk]))[0]) for tk in tok[pos:pos + n_p]]
            assert keys == sorted(keys, reverse=True)
            # nothing unselected in this patch is older than something selected
            members = [(t * cfg.height + y0 + dy) * cfg.width + x0 + dx for dy in range(hh) for dx in range(ww)]
            unsel = [m for m in members if m not in set(tok[pos:pos + n_p].tolist())]
            if unsel and n_p:
                assert max(ages[m] for m in unsel) <= min(ages[tk] for tk in tok[pos:pos + n_p])
            pos += n_p
        assert pos == len(idx)
        # age update: selected -> 0, others + 1
        want = ages + 1
        want[tok] = 0
        np.testing.assert_array_equal(new_ages, want)
        last_seen[tok] = step
        assert (step - last_seen).max() <= worst_wait                # bounded neglect
        assert new_ages.max() <= worst_wait - 1
        ages = new_ages
    # determinism
    a, _ = O.select(np.zeros(cfg.n_video, np.int32), cfg, 5)
    b, _ = O.select(np.zeros(cfg.n_video, np.int32), cfg, 5)
    np.testing.assert_array_equal(a, b)


def test_first_step_picks_are_uniform_within_patches():
    """With equal ages the rule is uniform random sampling: chi-square over the 4
    positions of a 2x2 patch, over many patches and steps."""
    cfg = get_config("cvx2b_block", frames=2, height=30, width=44)
    counts = np.zeros(4)
    for step in range(1, 9):
        idx, _ = O.select(np.zeros(cfg.n_video, np.int32), cfg, step)
        tok = idx.astype(int) - cfg.n_text
        y = (tok % (cfg.height * cfg.width)) // cfg.width
        x = tok % cfg.width
        np.add.at(counts, (y % 2) * 2 + (x % 2), 1)
    expected = counts.sum() / 4
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert chi2 < 16.27            # 3 dof, p = 0.001


def test_position_rotates_over_consecutive_cached_steps():
    cfg = get_config("tiny")
    ages = np.zeros(cfg.n_video, np.int32)
    seen = np.zeros(cfg.n_video, int)
    for step in (1, 2, 3, 4):
        idx, ages = O.select(ages, cfg, step)
        seen[idx - cfg.n_text] += 1
    assert (seen == 1).all()       # 2x2 patches, one per step: four steps visit every token once


# ---------------------------------------------------------------- age-weighted sampling (second reading of Sec. 3.3)

def exact_inclusion_probabilities(weights, n_take):
    """Inclusion probability of each item under sequential weighted sampling without
    replacement, by enumerating every ordered outcome (exact rational arithmetic)."""
    from fractions import Fraction
    n = len(weights)
    incl = [Fraction(0)] * n

    def rec(left, prob, depth):
        if depth == n_take:
            for e in range(n):
                if e not in left:
                    incl[e] += prob
            return
        total = sum(weights[e] for e in left)
        for e in left:
            rec(left - {e}, prob * Fraction(weights[e], total), depth + 1)
    rec(frozenset(range(n)), Fraction(1), 0)
    return [float(p) for p in incl]


def test_sample_weighted_maps_the_random_word_onto_the_running_sums():
    # weights 1,2,3 -> [0,1) item 0, [1,3) item 1, [3,6) item 2; r = floor(u * 6 / 2^32)
    w = [1, 2, 3]
    two32 = 1 << 32
    assert O.sample_weighted(w, 1, [0]) == [0]
    assert O.sample_weighted(w, 1, [two32 // 6 - 1]) == [0]
    assert O.sample_weighted(w, 1, [two32 // 6 + 1]) == [1]
    assert O.sample_weighted(w, 1, [two32 // 2 - 1]) == [1]
    assert O.sample_weighted(w, 1, [two32 // 2]) == [2]
    assert O.sample_weighted(w, 1, [two32 - 1]) == [2]
    # second draw works on what is left: after taking item 2, total 3: [0,1) item 0, [1,3) item 1
    assert O.sample_weighted(w, 2, [two32 - 1, 0]) == [2, 0]
    assert O.sample_weighted(w, 2, [two32 - 1, two32 // 3 + 1]) == [2, 1]
    assert sorted(O.sample_weighted(w, 3, [5, 7, 11])) == [0, 1, 2]       # taking everything


@pytest.mark.parametrize("n_take", [1, 2, 3])
def test_age_weighted_sampling_follows_the_exact_inclusion_probabilities(n_take):
    """2x3 patches whose six tokens have ages 0..5 (weights 1..6): the empirical inclusion
    frequencies over all patches and many steps match the enumerated probabilities of
    sequential weighted sampling without replacement."""
    cfg = get_config("paper_point", frames=2, ratio=n_take / 6.0, select_mode=1)
    assert O.tokens_per_patch(cfg.ratio, 6) == n_take
    tok = np.arange(cfg.n_video)
    y, x = (tok % (cfg.height * cfg.width)) // cfg.width, tok % cfg.width
    pos = (y % 2) * 3 + (x % 3)                       # position inside the 2x3 patch = its age
    ages = pos.astype(np.int32)
    counts = np.zeros(6)
    n_steps = 40
    for step in range(1, n_steps + 1):
        idx, _ = O.select(ages, cfg, step)
        np.add.at(counts, pos[idx.astype(int) - cfg.n_text], 1)
    n_patches = cfg.n_video // 6
    freq = counts / (n_patches * n_steps)
    want = np.array(exact_inclusion_probabilities([1, 2, 3, 4, 5, 6], n_take))
    assert abs(freq.sum() - n_take) < 1e-9
    sigma = np.sqrt(want * (1 - want) / (n_patches * n_steps))
    assert (np.abs(freq - want) < 4.5 * sigma + 1e-12).all(), (freq, want)
    assert (np.diff(freq) > 0).all()                  # neglected longer => more likely


def test_age_weighted_sampling_invariants_and_age_tail():
    cfg = get_config("tiny", height=7, width=9, patch_h=2, patch_w=3, ratio=0.34, select_mode=1)
    patches = O.patch_list(cfg.frames, cfg.height, cfg.width, cfg.patch_h, cfg.patch_w)
    ages = np.zeros(cfg.n_video, np.int32)
    old = 0
    for step in range(1, 61):
        idx, new_ages = O.select(ages, cfg, step)
        tok = idx.astype(int) - cfg.n_text
        assert len(np.unique(idx)) == len(idx) and tok.min() >= 0 and tok.max() < cfg.n_video
        p0 = 0
        for (t, y0, x0, hh, ww) in patches:
            n_p = O.tokens_per_patch(cfg.ratio, hh * ww)
            for tk in tok[p0:p0 + n_p]:
                tt, rem = divmod(tk, cfg.height * cfg.width)
                yy, xx = divmod(rem, cfg.width)
                assert tt == t and y0 <= yy < y0 + hh and x0 <= xx < x0 + ww
            p0 += n_p
        assert p0 == len(idx)
        want = ages + 1
        want[tok] = 0
        np.testing.assert_array_equal(new_ages, want)
        ages = new_ages
        if step > 20:
            old += int((ages >= 9).sum())
    # 2 of 6 per step: age-blind sampling leaves (2/3)^9 = 2.6 % of the tokens older than 8 steps;
    # weighting by age + 1 makes that far rarer
    assert old / (40 * cfg.n_video) < 0.004
    a, _ = O.select(np.zeros(cfg.n_video, np.int32), cfg, 5)
    b, _ = O.select(np.zeros(cfg.n_video, np.int32), cfg, 5)
    c, _ = O.select(np.zeros(cfg.n_video, np.int32), cfg.with_(seed=77), 5)
    np.testing.assert_array_equal(a, b)
    assert not np.array_equal(a, c)


def test_age_weighted_degenerate_cases():
    cfg = get_config("tiny", select_mode=1)
    idx, ages = O.select(np.full(cfg.n_video, 3, np.int32), cfg.with_(ratio=1.0), 2)
    assert sorted(idx.tolist()) == list(range(cfg.n_text, cfg.n_tokens)) and (ages == 0).all()
    idx, ages = O.select(np.full(cfg.n_video, 3, np.int32), cfg.with_(ratio=0.0), 2)
    assert len(idx) == 0 and (ages == 4).all()
    # one token overwhelmingly old: it is taken (weight 65536 against three of weight 1)
    a0 = np.zeros(cfg.n_video, np.int32)
    a0[5] = 10 ** 6
    hits = sum(int(cfg.n_text + 5 in O.select(a0, cfg, s)[0]) for s in range(1, 41))
    assert hits >= 39


# ---------------------------------------------------------------- cost model (Tables 1, 3, 4)

def test_cost_model_matches_paper_flops_structure():
    t1 = {r[0]: float(r[2]) for r in load_table("paper_table1_efficiency.txt")}
    t3 = [(float(r[0]), float(r[2])) for r in load_table("paper_table3_ratio_sweep.txt")]
    t4 = [(int(r[0]), float(r[2])) for r in load_table("paper_table4_threshold_sweep.txt")]

    # (i) M = 2 means one cached step per interval: the pure-reuse row costs 25 of 50 forwards
    fwd = (t1["full"] - t1["reuse_M2"]) / 25.0             # one DiT forward, T
    fixed = t1["full"] - 50 * fwd                           # work outside the block stack
    assert 250 < fwd < 280 and fixed > 0

    # (ii) Table 4 is linear in K
    ks = np.array([k for k, _ in t4], float)
    fl = np.array([f for _, f in t4])
    slope_k, icpt = np.polyfit(ks, fl, 1)
    assert np.abs(fl - (slope_k * ks + icpt)).max() < 0.2

    # (iii) Table 3 is linear in tokens-per-patch with zero intercept: n = 0 gives the pure-reuse row
    ns = np.array([O.tokens_per_patch(r, 6) for r, _ in t3], float)
    f3 = np.array([f for _, f in t3])
    slope_n, icpt_n = np.polyfit(ns, f3, 1)
    assert abs(icpt_n - t1["reuse_M2"]) < 1.0

    # (iv) one refreshed layer costs r/N of a full layer: queries against the FULL key set,
    #      no r^2 term.  Our model on the paper's operating point gives the same fraction.
    cfg = get_config("paper_point")
    per_layer_refresh = slope_k / 25.0                      # 25 cached steps
    frac_paper = per_layer_refresh / (fwd / cfg.n_layers)
    r = 2925
    frac_model = O.layer_flops(r, cfg.n_tokens, cfg.hidden, cfg.ffn_dim) / \
        O.layer_flops(cfg.n_tokens, cfg.n_tokens, cfg.hidden, cfg.ffn_dim)
    assert abs(frac_model - r / cfg.n_tokens) < 1e-12
    assert abs(frac_paper - frac_model) / frac_model < 0.01
    # a model with queries attending only to refreshed keys would be far off
    frac_r2 = O.layer_flops(r, r, cfg.hidden, cfg.ffn_dim) / \
        O.layer_flops(cfg.n_tokens, cfg.n_tokens, cfg.hidden, cfg.ffn_dim)
    assert abs(frac_paper - frac_r2) / frac_paper > 0.2

    # (v) schedule_flops has the same structure: linear in K, linear in r, zero intercept
    base = O.schedule_flops(cfg.with_(n_shallow=0), 50)
    assert base == 25 * cfg.n_layers * O.layer_flops(cfg.n_tokens, cfg.n_tokens, cfg.hidden, cfg.ffn_dim)
    s10 = O.schedule_flops(cfg.with_(n_shallow=10), 50) - base
    s20 = O.schedule_flops(cfg.with_(n_shallow=20), 50) - base
    assert abs(s20 - 2 * s10) / s20 < 1e-12
    r1 = O.schedule_flops(cfg, 50, refreshed_rows=1000) - base
    r2 = O.schedule_flops(cfg, 50, refreshed_rows=2000) - base
    assert abs(r2 - 2 * r1) / r2 < 1e-12
    assert O.schedule_flops(cfg, 50, refreshed_rows=0) == base
    # absolute scale: the paper does not state its token count; solving its per-layer cost
    # 24 N d^2 + 4 N^2 d = fwd/42 for N gives about 15.2k tokens, i.e. 11 latent frames of
    # 30x45 plus text.  At that size the model reproduces the per-K slope within 3 %.
    n_paper = (-18432 + math.sqrt(18432 ** 2 + 4 * (fwd / 42 * 1e12) / (4 * 3072))) / 2
    assert 14000 < n_paper < 16500
    cfg11 = cfg.with_(frames=11)
    b11 = O.schedule_flops(cfg11.with_(n_shallow=0), 50)
    s11 = (O.schedule_flops(cfg11.with_(n_shallow=10), 50) - b11) / 10 / 1e12
    assert abs(s11 - slope_k) / slope_k < 0.03
