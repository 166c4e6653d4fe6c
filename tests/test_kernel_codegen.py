"""Code-generation guard for the attention kernel (CPU only: hipcc cross-compiles to assembly).

The head_dim-64 kernel needs every vector register inside its key loop; a few instructions added
anywhere in the function have made the register allocator park a value in scratch memory inside
that loop, and the wait for its reload (which also waits for every outstanding K/V fill) cost
2-4 % of the kernel.  This test compiles the kernel and looks at the loop."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_17588_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_attention_key_loop_touches_no_scratch_memory():
    from paper_2508_17588_amd.build import FLAGS
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "attention.s")
        flags = [f for f in FLAGS if f != "-fPIC"]
        res = subprocess.run([HIPCC, *flags, "--cuda-device-only", "-S", os.path.join(CSRC, "attention.hip"), "-o", out],
                             capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]
        text = open(out).read()
    m = re.search(r"^(_Z\w*attention_hd64_kernelILi4E\w*):[^\n]*\n(.*?)s_endpgm", text, re.S | re.M)
    assert m, "attention_hd64_kernel<4> not found in the assembly"
    body = m.group(2).split("\n")
    # the key loop: the innermost loop with the most MFMAs
    loops, start = [], None
    for i, line in enumerate(body):
        if "Loop Header" in line:
            start = i
        elif start is not None and re.match(r"\s*s_cbranch_\w+\s+\.LBB", line):
            loops.append(body[start:i + 1])
            start = None
    assert loops, "no loop found"
    key_loop = max(loops, key=lambda l: sum("v_mfma" in x for x in l))
    ops = [x.split()[0] for x in key_loop if x.strip() and not x.strip().startswith((";", "."))]
    n_mfma = sum(o.startswith("v_mfma_f32_32x32x16_bf16") for o in ops)
    assert n_mfma == 96, f"key loop holds {n_mfma} MFMAs, expected 96 (three 64-key tiles)"
    scratch = [o for o in ops if o.startswith("scratch_") or o.startswith("buffer_store")]
    assert not scratch, f"key loop touches scratch memory: {scratch}"
    assert sum(o.startswith("v_exp_f32") for o in ops) == 192
