"""GPU parity of each kernel against the CPU oracle's matching routine, through the C ABI.

Integer work (selection, ages) must be bit-exact; bf16 activations must be within
max-abs 2e-2 and mean-relative 5e-3 of the float64 oracle on the same seeded inputs.
"""
import numpy as np
import pytest
import torch

from oracle import hero_oracle as O
from paper_2508_17588_amd import binding as B
from workloads import get_config, round_to_bf16
from hero_testlib import assert_close, to_dev_bf16, to_host_f64

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", flush=True)


def rnd(seed, *shape, scale=1.0):
    return round_to_bf16(np.random.default_rng(seed).standard_normal(shape, dtype=np.float32) * np.float32(scale))


# ---------------------------------------------------------------- selection

@pytest.mark.parametrize("name,over", [
    ("tiny", {}),
    ("tiny", dict(height=7, width=9, patch_h=2, patch_w=3, ratio=0.34)),
    ("tiny", dict(frames=2, height=5, width=5, patch_h=3, patch_w=2, ratio=0.5, seed=(7 << 32) | 99)),
    ("tiny", dict(ratio=1.0)),
    ("tiny", dict(ratio=0.0)),
    ("cvx2b_block", dict(hidden=64, n_heads=1, ffn_dim=64)),     # the real 13x30x45 grid, 2x2 clipped at x=44
    ("cvx2b_block", dict(hidden=64, n_heads=1, ffn_dim=64, patch_h=2, patch_w=5, ratio=0.1)),
    ("paper_point", dict(hidden=64, n_heads=1, ffn_dim=64, n_layers=1, n_shallow=1)),
    # age-weighted sampling without replacement (second reading of the tracking paragraph)
    ("tiny", dict(select_mode=1)),
    ("tiny", dict(select_mode=1, height=7, width=9, patch_h=2, patch_w=3, ratio=0.34)),
    ("tiny", dict(select_mode=1, frames=2, height=5, width=5, patch_h=3, patch_w=2, ratio=0.5, seed=(7 << 32) | 99)),
    ("tiny", dict(select_mode=1, ratio=1.0)),
    ("tiny", dict(select_mode=1, ratio=0.0)),
    ("tiny", dict(select_mode=1, patch_h=64, patch_w=64, ratio=0.3)),     # one clipped 8x8 patch per frame
    ("cvx2b_block", dict(select_mode=1, hidden=64, n_heads=1, ffn_dim=64)),
    ("paper_point", dict(select_mode=1, hidden=64, n_heads=1, ffn_dim=64, n_layers=1, n_shallow=1)),
    ("paper_point", dict(select_mode=1, hidden=64, n_heads=1, ffn_dim=64, n_layers=1, n_shallow=1, ratio=0.5)),
])
def test_select_bit_exact(name, over):
    cfg = get_config(name, **over)
    say(f"select {name} {over}")
    cache = B.HeroCache(B.make_config(cfg))
    n_sel = B.hero_num_selected(cache.cfg)
    idx = torch.full((max(n_sel, 1),), -1, dtype=torch.int32, device="cuda")
    ages = np.zeros(cfg.n_video, np.int32)
    for step in (1, 2, 3, 5, 6, 7, 9, 1000003):
        want_idx, ages = O.select(ages, cfg, step)
        got_n = cache.hero_select(step, idx)
        torch.cuda.synchronize()
        assert got_n == len(want_idx) == n_sel
        np.testing.assert_array_equal(idx[:n_sel].cpu().numpy(), want_idx)
        np.testing.assert_array_equal(cache.hero_cache_view(0, B.VIEW_AGES).cpu().numpy(), ages)
    cache.hero_reset_ages()
    torch.cuda.synchronize()
    assert int(cache.hero_cache_view(0, B.VIEW_AGES).abs().max().item()) == 0
    cache.close()


# ---------------------------------------------------------------- gather + LayerNorm

@pytest.mark.parametrize("hidden,x_dtype", [(128, torch.float32), (1920, torch.float32), (3072, torch.bfloat16),
                                            (3072, torch.float32), (8192, torch.float32), (72, torch.bfloat16)])
def test_gather_ln(hidden, x_dtype):
    say(f"gather_ln hidden={hidden} {x_dtype}")
    n = 301
    x = rnd(1, n, hidden, scale=2.0) + np.float32(0.5)
    x = round_to_bf16(x)
    add = rnd(2, n, hidden, scale=0.3)
    gain = round_to_bf16(1 + rnd(3, hidden, scale=0.2))
    bias = rnd(4, hidden, scale=0.2)
    rows = np.random.default_rng(5).permutation(n)[:157].astype(np.int32)
    xd = torch.from_numpy(x).cuda().to(x_dtype)
    out = torch.zeros(len(rows) + 3, hidden, dtype=torch.bfloat16, device="cuda")
    for use_add, use_rows in ((False, True), (True, True), (True, False)):
        rr = rows if use_rows else np.arange(n, dtype=np.int32)[:157]
        B.hero_gather_ln(xd, to_dev_bf16(add) if use_add else None,
                         torch.from_numpy(rr).cuda() if use_rows else None, len(rr),
                         to_dev_bf16(gain), to_dev_bf16(bias), 1e-5, out)
        torch.cuda.synchronize()
        src = x.astype(np.float64)[rr] + (add.astype(np.float64)[rr] if use_add else 0.0)
        want = O.layer_norm(src, gain.astype(np.float64), bias.astype(np.float64), 1e-5)
        assert_close(to_host_f64(out[:len(rr)]), want, f"gather_ln add={use_add} rows={use_rows}")
        assert float(out[len(rr):].abs().max()) == 0.0         # rows past n_rows untouched
    B.hero_gather_ln(xd, None, None, 0, to_dev_bf16(gain), to_dev_bf16(bias), 1e-5, out)   # empty is a no-op


# ---------------------------------------------------------------- linear (MFMA GEMM)

@pytest.mark.parametrize("m,n,k,act", [
    (1, 128, 64, 0), (300, 384, 128, 0), (64, 128, 512, 1), (257, 512, 128, 1),
    (1000, 1920, 256, 0), (3000, 3072, 256, 0), (3001, 3072 + 64, 192, 1), (4485, 5760, 128, 0),
    # large-tile kernel with 1, 5 and 7 stages of 64 (its stage loop is unrolled six times, the
    # activation ring is three slots deep)
    (4096, 2048, 64, 0), (3000, 3072, 320, 1), (3000, 3072, 448, 0),
])
def test_linear(m, n, k, act):
    say(f"linear m={m} n={n} k={k} act={act}")
    a = rnd(10, m, k)
    w = rnd(11, n, k, scale=1.0 / np.sqrt(k))
    b = rnd(12, n, scale=0.5)
    c = torch.full((m + 2, n), 7.0, dtype=torch.bfloat16, device="cuda")
    B.hero_linear(to_dev_bf16(a), to_dev_bf16(w), to_dev_bf16(b), c, act)
    torch.cuda.synchronize()
    want = O.linear(a.astype(np.float64), w.astype(np.float64), b.astype(np.float64))
    if act:
        want = O.gelu_tanh(want)
    assert_close(to_host_f64(c[:m]), want, "linear")
    assert float((c[m:] - 7.0).abs().max()) == 0.0              # rows past M untouched


@pytest.mark.parametrize("m,n,k,act,scratch_mib", [
    (2040, 4096, 4096, 0, 64),       # 128 tiles, all cut in two
    (2700, 6144, 6144, 1, 64),       # 264 tiles: 256 whole, 8 cut in six
    (2700, 6144, 6144, 0, 5),        # scratch for two chunks per tile only
    (2700, 6144, 6144, 0, 1),        # scratch too small to cut anything
    (2700, 6144, 1024, 0, 64),       # k too short to cut
    (4000, 3072, 3072, 0, 64),       # 192 tiles: the round is too full to cut
])
def test_linear_with_k_split(m, n, k, act, scratch_mib):
    say(f"linear (k-split) m={m} n={n} k={k} act={act} scratch={scratch_mib} MiB")
    a = rnd(13, m, k)
    w = rnd(14, n, k, scale=1.0 / np.sqrt(k))
    b = rnd(15, n, scale=0.5)
    c = torch.full((m + 2, n), 7.0, dtype=torch.bfloat16, device="cuda")
    scratch = torch.full((scratch_mib << 18,), float("nan"), dtype=torch.float32, device="cuda")
    B.hero_linear_scratch(to_dev_bf16(a), to_dev_bf16(w), to_dev_bf16(b), c, scratch, act)
    torch.cuda.synchronize()
    want = O.linear(a.astype(np.float64), w.astype(np.float64), b.astype(np.float64))
    if act:
        want = O.gelu_tanh(want)
    assert_close(to_host_f64(c[:m]), want, "linear with k-split")
    assert float((c[m:] - 7.0).abs().max()) == 0.0


def _random_linear_shapes():
    """Seeded shapes around the kernels' tile edges: both kernels, ragged m, every n and k granule."""
    g = np.random.default_rng(2024)
    shapes = []
    for _ in range(10):         # small-tile kernel
        shapes.append((int(g.integers(1, 1500)), 64 * int(g.integers(1, 20)), 64 * int(g.integers(1, 12))))
    for _ in range(8):          # at least 128 tiles of 256 x 256: large-tile kernel, 1 to 3 rounds
        tm, tn = int(g.integers(8, 30)), int(g.integers(8, 24))
        tn = max(tn, -(-128 // tm))
        shapes.append((256 * tm - int(g.integers(0, 255)), 256 * tn - 64 * int(g.integers(0, 4)), 64 * int(g.integers(1, 40))))
    return shapes


@pytest.mark.parametrize("m,n,k", _random_linear_shapes())
def test_linear_random_shapes(m, n, k):
    say(f"linear (random shape) m={m} n={n} k={k}")
    a = rnd(60, m, k)
    w = rnd(61, n, k, scale=1.0 / np.sqrt(k))
    b = rnd(62, n, scale=0.5)
    want = O.gelu_tanh(O.linear(a.astype(np.float64), w.astype(np.float64), b.astype(np.float64)))
    ad, wd, bd = to_dev_bf16(a), to_dev_bf16(w), to_dev_bf16(b)
    scratch = torch.full((64 << 18,), float("nan"), dtype=torch.float32, device="cuda")
    for use_scratch in (False, True):
        c = torch.full((m + 1, n), 9.0, dtype=torch.bfloat16, device="cuda")
        if use_scratch:
            B.hero_linear_scratch(ad, wd, bd, c, scratch, 1)
        else:
            B.hero_linear(ad, wd, bd, c, 1)
        torch.cuda.synchronize()
        assert_close(to_host_f64(c[:m]), want, f"linear random shape scratch={use_scratch}")
        assert float((c[m:] - 9.0).abs().max()) == 0.0


def test_empty_problems_are_no_ops():
    say("linear with m = 0, attention with r = 0, axpy with no elements")
    w, b = to_dev_bf16(rnd(16, 128, 64)), to_dev_bf16(rnd(17, 128))
    rows = torch.zeros(4, 64, dtype=torch.bfloat16, device="cuda")
    c = torch.full((2, 128), 5.0, dtype=torch.bfloat16, device="cuda")
    B.hero_linear(rows[:0], w, b, c, 0)
    scratch = torch.zeros(1 << 18, dtype=torch.float32, device="cuda")
    B.hero_linear_scratch(rows[:0], w, b, c, scratch, 1)
    k = to_dev_bf16(rnd(18, 64, 64))
    vt = to_dev_bf16(rnd(19, 64, 64))
    o = torch.full((2, 64), 5.0, dtype=torch.bfloat16, device="cuda")
    B.hero_attention(rows[:0], k, vt, o, 64, 1, 64)
    B.hero_attention(rows[:0], k, vt, o, 64, 1, 64, scratch)
    x = torch.full((16,), 5.0, dtype=torch.float32, device="cuda")
    B.hero_axpy_features(x[:0], c.reshape(-1)[:0], None, 0.0)
    torch.cuda.synchronize()
    assert float((c - 5.0).abs().max()) == 0.0 and float((o - 5.0).abs().max()) == 0.0
    assert float((x - 5.0).abs().max()) == 0.0


# ---------------------------------------------------------------- attention

def vt_padded(v, ld):
    vt = np.zeros((v.shape[1], ld), np.float32)
    vt[:, :v.shape[0]] = v.T
    return vt


@pytest.mark.parametrize("r,n_keys,heads,hd,case", [
    (1, 1, 1, 64, "plain"), (5, 11, 2, 64, "plain"), (64, 64, 1, 64, "plain"), (300, 1000, 3, 64, "plain"),
    (257, 129, 2, 32, "plain"), (70, 272, 4, 32, "plain"), (130, 777, 2, 64, "peaky"),
    (130, 777, 2, 64, "outlier"), (513, 2048, 1, 64, "plain"),
    # scores far outside the fp32 exponent range of a reference-free exp2: the head_dim-64 kernel
    # must notice and recompute with the running-maximum form (huge: overflow, allneg: every
    # probability underflows, onequery: a single query of the workgroup is affected)
    (130, 777, 2, 64, "huge"), (130, 777, 2, 64, "allneg"), (300, 200, 1, 64, "onequery"),
    (70, 272, 4, 32, "huge"),
])
def test_attention(r, n_keys, heads, hd, case):
    run_attention(r, n_keys, heads, hd, case, scratch_mib=0)


# query blocks cut along the keys (their partial sums pass through scratch): every block is cut here
# because the grid is far smaller than the chip; n_keys = 4133 has 64 whole key tiles and a ragged
# tail, so ranges of 16 tiles; 3000 keys: ranges of 23 / 23 tiles; 1 MiB of scratch: fewer ranges
@pytest.mark.parametrize("r,n_keys,heads,hd,case,scratch_mib", [
    (600, 4133, 4, 64, "plain", 64), (600, 4133, 4, 64, "peaky", 64), (600, 4133, 4, 64, "huge", 64),
    (600, 4133, 4, 64, "allneg", 64), (600, 4133, 4, 64, "onequery", 64), (257, 3000, 2, 64, "plain", 64),
    (600, 4133, 4, 64, "plain", 3), (600, 4133, 4, 64, "plain", 1), (300, 2048, 3, 32, "plain", 64),
])
def test_attention_with_key_split(r, n_keys, heads, hd, case, scratch_mib):
    run_attention(r, n_keys, heads, hd, case, scratch_mib)


def _random_attention_shapes():
    g = np.random.default_rng(77)
    out = []
    for i in range(12):
        hd = 64 if i % 3 else 32
        out.append((int(g.integers(1, 900)), int(g.integers(1, 5000)), int(g.integers(1, 5)), hd, 64 if i % 2 else 0))
    return out


@pytest.mark.parametrize("r,n_keys,heads,hd,scratch_mib", _random_attention_shapes())
def test_attention_random_shapes(r, n_keys, heads, hd, scratch_mib):
    run_attention(r, n_keys, heads, hd, "plain", scratch_mib)


def run_attention(r, n_keys, heads, hd, case, scratch_mib):
    say(f"attention r={r} n_keys={n_keys} heads={heads} hd={hd} {case} scratch={scratch_mib} MiB")
    d = heads * hd
    q, k, v = rnd(20, r, d), rnd(21, n_keys, d), rnd(22, n_keys, d)
    if case == "peaky":
        q, k = round_to_bf16(q * 4), round_to_bf16(k * 4)
    if case == "outlier":
        k[3] = round_to_bf16(k[3] * 50)
    if case == "huge":
        q = round_to_bf16(q * 64)
    if case == "allneg":
        k[:, ::hd] = 16.0           # channel 0 of every head: all keys share a large component ...
        q[:, ::hd] = -128.0         # ... that every query opposes: all scores ~ -2048/sqrt(hd)
    if case == "onequery":
        q[77] = round_to_bf16(q[77] * 200)
    ld = (n_keys + 63) // 64 * 64
    o = torch.full((r + 1, d), 3.0, dtype=torch.bfloat16, device="cuda")
    scratch = (torch.full((scratch_mib << 18,), float("nan"), dtype=torch.float32, device="cuda")
               if scratch_mib else None)
    fallbacks = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.hero_attention(to_dev_bf16(q), to_dev_bf16(k), to_dev_bf16(vt_padded(v, ld)), o, n_keys, heads, hd, scratch, fallbacks)
    torch.cuda.synchronize()
    want = O.attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), heads)
    assert_close(to_host_f64(o[:r]), want, "attention")
    assert float((o[r:] - 3.0).abs().max()) == 0.0
    # how many workgroups (256 queries of one head) left the maximum-free path is counted
    n_wg = (r + 255) // 256 * heads
    # (peaky and outlier scores reach the edge of the maximum-free range: some workgroups may leave it)
    expect = {"plain": 0, "huge": n_wg, "allneg": n_wg, "onequery": heads}.get(case) if hd == 64 else 0
    if expect is not None:
        assert int(fallbacks.item()) == expect, (int(fallbacks.item()), expect)


def test_attention_key_count_smaller_than_buffer():
    """Keys beyond n_keys in the K buffer and the V^T padding must not leak in."""
    say("attention n_keys < rows of the K buffer")
    r, n_keys, heads, hd = 40, 100, 2, 64
    d = heads * hd
    q, k, v = rnd(30, r, d), rnd(31, 128, d), rnd(32, 128, d)
    vt = vt_padded(v, 128)
    vt[:, n_keys:] = 0.0
    o = torch.zeros(r, d, dtype=torch.bfloat16, device="cuda")
    B.hero_attention(to_dev_bf16(q), to_dev_bf16(k), to_dev_bf16(vt), o, n_keys, heads, hd)
    torch.cuda.synchronize()
    want = O.attention(q.astype(np.float64), k[:n_keys].astype(np.float64), v[:n_keys].astype(np.float64), heads)
    assert_close(to_host_f64(o), want, "attention (short key count)")


# ---------------------------------------------------------------- residual / extrapolation update

@pytest.mark.parametrize("x_dtype", [torch.float32, torch.bfloat16])
def test_axpy_features(x_dtype):
    say(f"axpy_features {x_dtype}")
    n, d = 1001, 1920
    x, cur, prev = rnd(40, n, d), rnd(41, n, d, scale=0.3), rnd(42, n, d, scale=0.3)
    for alpha, use_prev in ((0.0, False), (0.25, True), (0.75, True), (0.0, True), (1.0, True)):
        xd = torch.from_numpy(x).cuda().to(x_dtype)
        B.hero_axpy_features(xd, to_dev_bf16(cur), to_dev_bf16(prev) if use_prev else None, alpha)
        torch.cuda.synchronize()
        c64, p64 = cur.astype(np.float64), prev.astype(np.float64)
        want = x.astype(np.float64) + (c64 + (c64 - p64) * alpha if use_prev else c64)
        got = to_host_f64(xd)
        if x_dtype == torch.float32:
            np.testing.assert_allclose(got, want, rtol=0, atol=2e-6)
        else:
            assert_close(got, want, "axpy bf16")
    # closed form (Eq. 5): features linear in the step are extrapolated exactly
    a, b = rnd(43, 64, 64), rnd(44, 64, 64, scale=0.125)
    g = lambda s: round_to_bf16(a + b * np.float32(s))
    xd = torch.zeros(64, 64, dtype=torch.float32, device="cuda")
    B.hero_axpy_features(xd, to_dev_bf16(g(8)), to_dev_bf16(g(4)), 3 / 4)
    torch.cuda.synchronize()
    want = g(8).astype(np.float64) + (g(8).astype(np.float64) - g(4).astype(np.float64)) * 0.75
    np.testing.assert_allclose(to_host_f64(xd), want, rtol=0, atol=1e-6)


# ---------------------------------------------------------------- stability statistics (Sec. 3.2)

@pytest.mark.parametrize("n,steps", [(8, 3), (4096 + 8, 3), (300 * 1920, 5), (17776 * 3072, 3)])
def test_second_diff_stats(n, steps):
    say(f"second-difference statistics n={n} steps={steps}")
    rng = np.random.default_rng(21)
    feats = [round_to_bf16((rng.standard_normal(n) * (0.5 + 0.2 * t)).astype(np.float32)) for t in range(steps)]
    dev = [to_dev_bf16(f) for f in feats]
    scratch = torch.empty(2048, dtype=torch.float64, device="cuda")
    stats = torch.full((2,), 123.0, dtype=torch.float64, device="cuda")
    for t in range(1, steps - 1):
        B.hero_second_diff_stats(dev[t - 1], dev[t], dev[t + 1], scratch, stats, accumulate=(t > 1))
    torch.cuda.synchronize()
    s1, s2 = stats.cpu().numpy()
    d = np.concatenate([feats[t + 1].astype(np.float64) - 2.0 * feats[t] + feats[t - 1] for t in range(1, steps - 1)])
    assert abs(s1 - d.sum()) <= 1e-11 * np.abs(d).sum()
    assert abs(s2 - (d * d).sum()) <= 1e-11 * (d * d).sum()
    cnt = d.size
    var = s2 / cnt - (s1 / cnt) ** 2
    np.testing.assert_allclose(var, O.second_difference_variance(feats), rtol=1e-9)
