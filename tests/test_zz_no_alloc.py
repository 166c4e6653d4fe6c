"""hero_linear_static: the GEMM with its k-split partial sums in the library's own device array
(for callers that cannot allocate), called through the C ABI and compared with
hero_linear_scratch, the entry point it is a variant of, and with the oracle.

Two calls in a row on the same device share the array; the second is a smaller problem, so parts
of the array still hold the first call's partial sums when it runs."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import hero_oracle as O
from paper_2508_17588_amd import binding as B
from hero_testlib import assert_close, to_dev_bf16, to_host_f64

pytestmark = pytest.mark.gpu

STATIC_BYTES = 32 << 20


def say(msg):
    print(f"[case] {msg}", flush=True)


def rnd(seed, *shape, scale=1.0):
    from workloads import round_to_bf16
    return round_to_bf16(np.random.default_rng(seed).standard_normal(shape, dtype=np.float32) * np.float32(scale))


def run_pair(m, n, k, act, seed):
    """-> (static result, scratch result, oracle rows, probe) for one problem."""
    a, w, b = rnd(seed, m, k), rnd(seed + 1, n, k, scale=1.0 / np.sqrt(k)), rnd(seed + 2, n, scale=0.5)
    ad, wd, bd = to_dev_bf16(a), to_dev_bf16(w), to_dev_bf16(b)
    c_static = torch.full((m + 2, n), 7.0, dtype=torch.bfloat16, device="cuda")
    c_scratch = torch.full((m + 2, n), 7.0, dtype=torch.bfloat16, device="cuda")
    scratch = torch.full((STATIC_BYTES // 4,), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    B.hero_linear_static(ad, wd, bd, c_static, act)
    B.hero_linear_scratch(ad, wd, bd, c_scratch, scratch, act)
    torch.cuda.synchronize()
    probe = np.unique(np.concatenate([np.random.default_rng(seed).choice(m, 200, replace=False), [0, m - 1]]))
    want = O.linear(a[probe].astype(np.float64), w.astype(np.float64), b.astype(np.float64))
    if act:
        want = O.gelu_tanh(want)
    return c_static, c_scratch, want, probe


def test_static_scratch_gemm_matches_the_caller_scratch_gemm_on_two_calls_in_a_row():
    # 296 tiles of 256 x 256: one round of 256 plus 40 tiles cut into 3 k-chunks (30 MiB of partial sums),
    # then 272 tiles: 16 cut in 2 (8 MiB), then a problem too small to be cut at all
    for (m, n, k, act, seed) in ((9472, 2048, 3072, 1, 100), (4300, 4096, 2048, 0, 200), (300, 256, 128, 1, 300)):
        say(f"hero_linear_static m={m} n={n} k={k} act={act}")
        c_static, c_scratch, want, probe = run_pair(m, n, k, act, seed)
        assert torch.equal(c_static, c_scratch), "static and caller scratch differ"      # same cut, same order of additions
        assert float((c_static[m:] - 7.0).abs().max()) == 0.0                         # rows past M untouched
        assert_close(to_host_f64(c_static[probe]), want, f"hero_linear_static {m}x{n}x{k} vs oracle")


def test_static_scratch_gemm_refuses_what_does_not_fit():
    say("hero_linear_static with a k-split that wants 54 MiB")
    lib = B.load_library()
    c = torch.full((8, 64), 3.0, dtype=torch.bfloat16, device="cuda")
    p = ctypes.c_void_p(c.data_ptr())
    # 840 tiles: 3 rounds and 72 tiles cut in 3 = 216 blocks of 256 KiB
    assert lib.hero_linear_static(p, p, p, p, 17776, 3072, 12288, 0, None) == B.HERO_ERR_BUFFER_TOO_SMALL
    assert b"hero_linear_scratch" in lib.hero_last_error()
    torch.cuda.synchronize()
    assert float((c - 3.0).abs().max()) == 0.0
