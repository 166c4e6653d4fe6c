"""Sizes at the edge of what the kernels accept.

The GEMM and attention kernels address their operands with 32-bit byte offsets; the launchers
accept a problem only while every offset a tile can form (rows past the end included) stays below
2^32.  These tests run each kernel just inside that bound, where the last rows sit within a few
MB of the 4 GiB mark, and compare sampled rows with the CPU oracle on the same seeded inputs; just
outside the bound the call must return an error without launching anything.
"""
import numpy as np
import pytest
import torch

from oracle import hero_oracle as O
from paper_2508_17588_amd import binding as B
from hero_testlib import assert_close, to_host_f64

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", flush=True)


def dev_randn_bf16(seed, rows, cols, scale=1.0):
    """Seeded N(0, scale) bf16 array drawn on the device in row blocks (no fp32 copy of the whole)."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    out = torch.empty(rows, cols, dtype=torch.bfloat16, device="cuda")
    step = max(1, (1 << 27) // cols)
    for i in range(0, rows, step):
        n = min(step, rows - i)
        out[i:i + n] = (torch.randn(n, cols, generator=gen, device="cuda") * scale).to(torch.bfloat16)
    return out


def rows_f64(t, rows):
    return to_host_f64(t[torch.as_tensor(rows, device="cuda")])


@pytest.mark.parametrize("m,n,k,kernel", [
    # (m + 512) * k * 2 = 4 291 657 728 < 2^32: 2727 row tiles of the 256 x 256 kernel
    (698_000, 256, 3072, "large-tile"),
    # 118 tiles of 256 x 256 is below the large-tile threshold: the 128 x 128 kernel, 1099 k steps
    (30_000, 128, 70_336, "small-tile"),
])
def test_linear_near_offset_limit(m, n, k, kernel):
    say(f"linear near the 32-bit offset limit ({kernel}) m={m} n={n} k={k}")
    assert (m + 512) * k * 2 < 2 ** 32
    a = dev_randn_bf16(40, m, k)
    w = dev_randn_bf16(41, n, k, scale=1.0 / np.sqrt(k))
    b = dev_randn_bf16(42, 1, n, scale=0.5).reshape(n)
    c = torch.full((m + 2, n), 1000.0, dtype=torch.bfloat16, device="cuda")
    B.hero_linear(a, w, b, c, 0)
    torch.cuda.synchronize()
    rows = sorted({0, 1, 127, 128, 255, 256, m // 2, m - 257, m - 256, m - 129, m - 2, m - 1})
    want = O.linear(rows_f64(a, rows), to_host_f64(w), to_host_f64(b))
    assert_close(rows_f64(c, rows), want, f"linear ({kernel}) sampled rows")
    assert float((c[m:] - 1000.0).abs().max()) == 0.0           # rows past M untouched
    assert float(c[:m].float().abs().max()) < 100.0             # every row was written (the fill value is gone)


def test_linear_beyond_offset_limit_is_an_error():
    m, n, k = 699_051, 256, 3072
    say(f"linear beyond the 32-bit offset limit m={m} k={k}")
    assert (m + 512) * k * 2 >= 2 ** 32
    a = torch.empty(m, k, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(n, k, dtype=torch.bfloat16, device="cuda")
    b = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    c = torch.full((m, n), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.HeroError):
        B.hero_linear(a, w, b, c, 0)
    torch.cuda.synchronize()
    assert float((c - 7.0).abs().max()) == 0.0                  # nothing ran


@pytest.mark.parametrize("scratch_mib", [0, 64])
def test_attention_near_offset_limit(scratch_mib):
    """698 500 keys of 48 heads x 64: K and V^T are 4.29 GB each; with scratch the query blocks are cut
    into key ranges, whose first keys then sit anywhere in that span."""
    r, n_keys, heads, hd = 300, 698_500, 48, 64
    d = heads * hd
    ld = (n_keys + 63) // 64 * 64
    say(f"attention near the 32-bit offset limit r={r} n_keys={n_keys} heads={heads} scratch={scratch_mib} MiB")
    assert (n_keys + 256) * d * 2 < 2 ** 32 and d * ld * 2 < 2 ** 32
    q = dev_randn_bf16(50, r, d)
    k = dev_randn_bf16(51, n_keys, d)
    vt = dev_randn_bf16(52, d, ld)
    vt[:, n_keys:] = 0
    o = torch.full((r + 1, d), 1000.0, dtype=torch.bfloat16, device="cuda")
    scratch = (torch.full((scratch_mib << 18,), float("nan"), dtype=torch.float32, device="cuda")
               if scratch_mib else None)
    B.hero_attention(q, k, vt, o, n_keys, heads, hd, scratch)
    torch.cuda.synchronize()
    queries = [0, 1, 63, 64, 255, 256, r - 2, r - 1]
    for head in (0, 23, heads - 1):
        cols = slice(head * hd, (head + 1) * hd)
        qh = rows_f64(q, queries)[:, cols]
        kh = to_host_f64(k[:, cols])
        vh = to_host_f64(vt[cols, :n_keys]).T
        want = O.attention(qh, kh, vh, 1)
        assert_close(rows_f64(o, queries)[:, cols], want, f"attention head {head}")
    assert float((o[r:] - 1000.0).abs().max()) == 0.0
    assert float(o[:r].float().abs().max()) < 100.0             # every output row was written


def test_attention_beyond_offset_limit_is_an_error():
    r, n_keys, heads, hd = 64, 699_100, 48, 64
    d = heads * hd
    ld = (n_keys + 63) // 64 * 64
    say(f"attention beyond the 32-bit offset limit n_keys={n_keys}")
    assert (n_keys + 256) * d * 2 >= 2 ** 32
    q = torch.zeros(r, d, dtype=torch.bfloat16, device="cuda")
    k = torch.empty(n_keys, d, dtype=torch.bfloat16, device="cuda")
    vt = torch.empty(d, ld, dtype=torch.bfloat16, device="cuda")
    o = torch.full((r, d), 3.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.HeroError):
        B.hero_attention(q, k, vt, o, n_keys, heads, hd)
    torch.cuda.synchronize()
    assert float((o - 3.0).abs().max()) == 0.0
