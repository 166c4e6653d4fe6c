"""Do the oracle's pins notice a mistake?

Each case plants one plausible mistake in the CPU oracle (a dropped term, a wrong sign, a
transposed or unscaled operand, a wrong rounding rule) by replacing one of its functions, then
runs the pin tests that are meant to guard that function: at least one of them must fail.  The
mistakes live here, in a CPU test; nothing on the GPU side is touched.
"""
import math

import numpy as np
import pytest

from oracle import hero_oracle as O

import test_oracle_components as TC
import test_oracle_layers as TL
import test_oracle_modblock as TM
import test_oracle_select as TS


# ----------------------------------------------------------------------------- the mistakes

def ln_unbiased_variance(x, gain, bias, eps):
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).sum(axis=-1, keepdims=True) / (x.shape[-1] - 1)
    return (x - mean) / np.sqrt(var + eps) * gain + bias


def ln_eps_outside_the_root(x, gain, bias, eps):
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    return (x - mean) / (np.sqrt(var) + eps) * gain + bias


def ln_gain_and_bias_swapped(x, gain, bias, eps):
    mean = x.mean(axis=-1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=-1, keepdims=True)
    return (x - mean) / np.sqrt(var + eps) * bias + gain


def gelu_erf_form(x):
    return 0.5 * x * (1.0 + np.vectorize(math.erf)(x / math.sqrt(2.0)))


def gelu_wrong_cubic_constant(x):
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.04715 * x ** 3)))


def linear_without_bias(x, w, b):
    return x @ w.T


def linear_untransposed(x, w, b):
    return x @ w + b          # only runs at all where W is square


def _attention(q, k, v, n_heads, scale=None, subtract_max=True, per_head=True, normalise=True):
    r, d = q.shape
    hd = d // n_heads
    out = np.empty_like(q)
    heads = range(n_heads) if per_head else [None]
    for h in heads:
        sl = slice(h * hd, (h + 1) * hd) if per_head else slice(0, d)
        s = (q[:, sl] @ k[:, sl].T) * (scale(hd) if scale else 1.0 / math.sqrt(hd))
        if subtract_max:
            s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        if normalise:
            p /= p.sum(axis=1, keepdims=True)
        out[:, sl] = p @ v[:, sl]
    return out


def attention_scaled_by_head_dim(q, k, v, n_heads):
    return _attention(q, k, v, n_heads, scale=lambda hd: 1.0 / hd)


def attention_unscaled(q, k, v, n_heads):
    return _attention(q, k, v, n_heads, scale=lambda hd: 1.0)


def attention_heads_not_split(q, k, v, n_heads):
    return _attention(q, k, v, n_heads, scale=lambda hd: 1.0 / math.sqrt(q.shape[1] // n_heads), per_head=False)


def attention_softmax_over_queries(q, k, v, n_heads):
    r, d = q.shape
    hd = d // n_heads
    out = np.empty_like(q)
    for h in range(n_heads):
        sl = slice(h * hd, (h + 1) * hd)
        s = (q[:, sl] @ k[:, sl].T) / math.sqrt(hd)
        p = np.exp(s - s.max(axis=0, keepdims=True))
        p /= p.sum(axis=0, keepdims=True)
        out[:, sl] = p @ v[:, sl]
    return out


def extrapolated_wrong_sign(cur, prev, k, interval):
    return cur.copy() if prev is None else cur - (cur - prev) * (k / interval)


def extrapolated_ratio_inverted(cur, prev, k, interval):
    return cur.copy() if prev is None else cur + (cur - prev) * (interval / max(k, 1))


def extrapolated_from_the_older_generation(cur, prev, k, interval):
    return cur.copy() if prev is None else prev + (cur - prev) * (k / interval)


def extrapolate_attention_branch_only(x, cache, k, interval):
    return x + O.extrapolated(cache.g_attn, cache.g_attn_prev, k, interval) + cache.g_ffn


def _refresh(x, w, cache, idx, n_heads, eps, write_kv_first=True, ffn_sees_attention=True, merge=True):
    d = x.shape[1]
    idx = np.asarray(idx, dtype=np.int64)
    if len(idx):
        u = O.layer_norm(x[idx], w["ln1_g"], w["ln1_b"], eps)
        qkv = O.linear(u, w["w_qkv"], w["b_qkv"])
        q, k, v = qkv[:, :d], qkv[:, d:2 * d], qkv[:, 2 * d:]
        if write_kv_first:
            cache.k[idx], cache.v[idx] = k, v
        g_attn = O.linear(O.attention(q, cache.k, cache.v, n_heads), w["w_o"], w["b_o"])
        if not write_kv_first:
            cache.k[idx], cache.v[idx] = k, v
        if merge:
            cache.g_attn[idx] = g_attn
        a = x[idx] + g_attn if ffn_sees_attention else x[idx]
        g_ffn = O.ffn(O.layer_norm(a, w["ln2_g"], w["ln2_b"], eps), w)
        if merge:
            cache.g_ffn[idx] = g_ffn
    return x + cache.g_attn + cache.g_ffn


def refresh_attends_to_stale_keys(x, w, cache, idx, n_heads, eps):
    return _refresh(x, w, cache, idx, n_heads, eps, write_kv_first=False)


def refresh_ffn_skips_the_attention_residual(x, w, cache, idx, n_heads, eps):
    return _refresh(x, w, cache, idx, n_heads, eps, ffn_sees_attention=False)


def refresh_does_not_merge_into_the_cache(x, w, cache, idx, n_heads, eps):
    return _refresh(x, w, cache, idx, n_heads, eps, merge=False)


def tokens_per_patch_floor(ratio, size):
    r = float(np.float32(ratio))
    return 0 if r <= 0.0 else int(min(max(math.floor(r * size), 1), size))


def tokens_per_patch_ceil(ratio, size):
    r = float(np.float32(ratio))
    return 0 if r <= 0.0 else int(min(max(math.ceil(r * size), 1), size))


def _select_with(age_rule):
    real = O.select

    def select(ages, cfg, step):
        idx, new_ages = real(ages, cfg, step)
        return idx, age_rule(np.asarray(ages, np.int64), idx.astype(np.int64) - cfg.n_text, new_ages)
    return select


select_keeps_the_age_of_sampled_tokens = _select_with(
    lambda ages, sel, new: (ages + 1).astype(np.int32))
select_never_ages_the_others = _select_with(
    lambda ages, sel, new: np.where(np.isin(np.arange(len(ages)), sel), 0, ages).astype(np.int32))
select_keeps_the_age_of_sampled_tokens.__name__ = "select_keeps_the_age_of_sampled_tokens"
select_never_ages_the_others.__name__ = "select_never_ages_the_others"


def select_ignores_ages(ages, cfg, step):
    return select_ignores_ages.real(np.zeros_like(np.asarray(ages)), cfg, step)[0], \
        select_ignores_ages.real(ages, cfg, step)[1]


select_ignores_ages.real = O.select


def second_difference_is_a_first_difference(features):
    f = [np.asarray(a, dtype=np.float64) for a in features]
    d = np.concatenate([(f[t + 1] - f[t]).ravel() for t in range(len(f) - 1)])
    return float(np.mean((d - d.mean()) ** 2))


def second_difference_second_moment(features):
    f = [np.asarray(a, dtype=np.float64) for a in features]
    d = np.concatenate([(f[t + 1] - 2.0 * f[t] + f[t - 1]).ravel() for t in range(1, len(f) - 1)])
    return float(np.mean(d ** 2))


def stability_not_inverted(variances):
    v = np.asarray(variances, dtype=np.float64)
    return np.ones_like(v) if v.max() == v.min() else (v - v.min()) / (v.max() - v.min())


def rope_turns_the_other_way(x, angles, n_heads):
    return O_apply_rope(x, -angles, n_heads)


def rope_pairs_split_in_halves(x, angles, n_heads):
    r, d = x.shape
    hd = d // n_heads
    xh = x.reshape(r, n_heads, hd)
    a, b = xh[..., :hd // 2], xh[..., hd // 2:]
    c, s_ = np.cos(angles)[:, None, :], np.sin(angles)[:, None, :]
    return np.concatenate([a * c - b * s_, a * s_ + b * c], axis=-1).reshape(r, d)


def rope_angles_one_frequency_per_axis(frames, height, width, head_dim):
    real = O_rope_angles(frames, height, width, head_dim)
    n_t, n_y = head_dim // 8, (head_dim // 16) * 3
    out = real.copy()
    out[:, :n_t] = real[:, :1]
    out[:, n_t:n_t + n_y] = real[:, n_t:n_t + 1]
    out[:, n_t + n_y:] = real[:, n_t + n_y:n_t + n_y + 1]
    return out


def head_layer_norm_over_the_whole_row(x, gain, bias, n_heads):
    hd = x.shape[1] // n_heads
    return O.layer_norm(x, np.tile(gain, n_heads), np.tile(bias, n_heads), O.QK_NORM_EPS)


O_apply_rope, O_rope_angles = O.apply_rope, O.rope_angles


# ----------------------------------------------------------------------------- the guards

def brute(case):
    return lambda: TC.test_attention_brute_force(case)


def sel_inv(i):
    params = TS.test_selection_invariants.pytestmark[0].args[1]
    return lambda: TS.test_selection_invariants(*params[i])


def refresh_is_full(flags):
    return lambda: TM.test_refresh_of_all_rows_is_the_full_layer_and_refresh_is_local(flags)


CASES = [
    ("layer_norm", ln_unbiased_variance, [TC.test_layer_norm_matches_library_and_closed_form]),
    ("layer_norm", ln_eps_outside_the_root, [TC.test_layer_norm_matches_library_and_closed_form]),
    ("layer_norm", ln_gain_and_bias_swapped, [TC.test_layer_norm_matches_library_and_closed_form]),
    ("gelu_tanh", gelu_erf_form, [TC.test_gelu_tanh_matches_library_and_limits]),
    ("gelu_tanh", gelu_wrong_cubic_constant, [TC.test_gelu_tanh_matches_library_and_limits]),
    ("linear", linear_without_bias, [TC.test_linear_matches_library_and_catches_transpose]),
    ("linear", linear_untransposed, [TC.test_linear_matches_library_and_catches_transpose]),
    ("attention", attention_scaled_by_head_dim, [brute("plain"), TC.test_attention_matches_library_sdpa]),
    ("attention", attention_unscaled, [brute("plain")]),
    ("attention", attention_heads_not_split, [brute("plain")]),
    ("attention", attention_softmax_over_queries, [brute("plain"), TC.test_attention_special_cases]),
    ("extrapolated", extrapolated_wrong_sign, [TL.test_p2_extrapolation_closed_form]),
    ("extrapolated", extrapolated_ratio_inverted, [TL.test_p2_extrapolation_closed_form]),
    ("extrapolated", extrapolated_from_the_older_generation, [TL.test_p2_extrapolation_closed_form]),
    ("extrapolate_layer", extrapolate_attention_branch_only, [TL.test_p2_extrapolate_layer_adds_both_branches]),
    ("refresh_layer", refresh_attends_to_stale_keys,
     [TL.test_p1_refresh_all_rows_equals_full_forward, TL.test_p4_refreshed_queries_see_refreshed_keys]),
    ("refresh_layer", refresh_ffn_skips_the_attention_residual, [TL.test_p1_refresh_all_rows_equals_full_forward]),
    ("refresh_layer", refresh_does_not_merge_into_the_cache,
     [TL.test_p1_refresh_all_rows_equals_full_forward, TL.test_p4_locality]),
    ("tokens_per_patch", tokens_per_patch_floor, [TS.test_tokens_per_patch_rounding_matches_table3_spacing]),
    ("tokens_per_patch", tokens_per_patch_ceil, [TS.test_tokens_per_patch_rounding_matches_table3_spacing]),
    ("select", select_keeps_the_age_of_sampled_tokens, [sel_inv(0), TS.test_position_rotates_over_consecutive_cached_steps]),
    ("select", select_never_ages_the_others, [sel_inv(0), TS.test_position_rotates_over_consecutive_cached_steps]),
    ("select", select_ignores_ages, [sel_inv(0), TS.test_position_rotates_over_consecutive_cached_steps]),
    ("second_difference_variance", second_difference_is_a_first_difference,
     [TC.test_second_difference_variance_closed_forms]),
    ("second_difference_variance", second_difference_second_moment,
     [TC.test_second_difference_variance_closed_forms]),
    ("stability_scores", stability_not_inverted, [TC.test_stability_scores_normalise_and_invert]),
    ("apply_rope", rope_turns_the_other_way,
     [TM.test_rope_is_a_rotation_and_depends_on_relative_position_only, TM.test_rope_angles_hand_computed]),
    ("apply_rope", rope_pairs_split_in_halves,
     [TM.test_rope_is_a_rotation_and_depends_on_relative_position_only, TM.test_text_rows_are_not_rotated_and_video_rows_are]),
    ("rope_angles", rope_angles_one_frequency_per_axis, [TM.test_rope_angles_hand_computed]),
    ("head_layer_norm", head_layer_norm_over_the_whole_row,
     [TM.test_head_layer_norm_is_the_library_layer_norm_per_head]),
]


@pytest.mark.parametrize("target,mistake,guards", CASES, ids=[c[1].__name__ for c in CASES])
def test_a_planted_mistake_fails_a_pin(monkeypatch, target, mistake, guards):
    for g in guards:                      # the guards pass on the oracle as it stands
        g()
    monkeypatch.setattr(O, target, mistake)
    caught = []
    for g in guards:
        try:
            g()
        except Exception as e:            # an assertion, or a shape error the mistake provokes
            caught.append(type(e).__name__)
    assert caught, f"no pin noticed {mistake.__name__} planted in oracle.{target}"
