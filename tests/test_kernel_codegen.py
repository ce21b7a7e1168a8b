"""Static checks of the generated gfx950 code of the two matrix-core kernels (no GPU needed: hipcc cross-compiles).

The contraction kernel feeds its pipeline with direct-to-LDS loads written as inline assembly, which the
compiler's wait-count bookkeeping does not see.  If register allocation ever places the reload of a spilled
register inside the contraction loop, the compiler guards it with `s_waitcnt vmcnt(0)`, which also drains
every load of the pipeline: the kernel stays correct and loses 40 % of its speed without any test failing.
These checks read the assembly and fail on that pattern.
"""
import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2503_01066_amd import build as B


def _device_asm(src):
    cmd = [B._hipcc()] + [f for f in B.FLAGS if f != "-fPIC"] + ["--cuda-device-only", "-S", os.path.join(B.CSRC, src), "-o", "-"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return r.stdout


@pytest.fixture(scope="module")
def asm():
    if not (shutil.which(B._hipcc()) or os.path.exists(B._hipcc())):
        pytest.skip("hipcc not found")
    with ThreadPoolExecutor(max_workers=2) as ex:
        texts = list(ex.map(_device_asm, ["gemm_mfma.hip", "attn_mfma.hip"]))
    return dict(zip(["gemm", "attn"], texts))


def _functions(text, prefix):
    for m in re.finditer(r"^(%s\w*):[^\n]*\n(.*?)^\.Lfunc_end" % prefix, text, re.S | re.M):
        yield m.group(1), m.group(2)


def _blocks(body):
    parts = re.split(r"^(\.LBB\d+_\d+):", body, flags=re.M)
    for i in range(1, len(parts), 2):
        yield parts[i], parts[i + 1]


def _meta(text, name, key):
    # one metadata entry per kernel, "  - .agpr_count: ..." first, keys in alphabetical order
    for entry in re.split(r"^  - \.agpr_count:", text, flags=re.M)[1:]:
        if re.search(r"\.name:\s+%s\n" % re.escape(name), entry):
            return int(re.search(r"\.%s:\s+(\d+)" % key, entry).group(1))
    raise AssertionError("no metadata for " + name)


def test_contraction_loops_hold_no_spill_code_and_no_full_wait(asm):
    seen = 0
    for name, body in _functions(asm["gemm"], "_ZN4alch11k_gemm_mfma"):
        loops = [(lab, txt) for lab, txt in _blocks(body) if txt.count("v_mfma_") >= 16]
        assert loops, name
        for lab, txt in loops:
            assert "scratch_" not in txt, "%s %s: spill code inside a contraction loop" % (name, lab)
            waits = re.findall(r"s_waitcnt ([^\n]*)", txt)
            assert not [w for w in waits if "vmcnt(0)" in w], "%s %s: the loop drains its load pipeline (%s)" % (name, lab, waits)
        seen += 1
    assert seen == 8  # four operand layouts, whole tiles and tiles split along the contraction


def test_attention_kernels_do_not_spill(asm):
    names = [n for n, _ in _functions(asm["attn"], "_ZN4alch")]
    kernels = [n for n in names if "k_attn_" in n]
    assert len(kernels) == 4, kernels  # dQ, dK/dV with and without prefixes, forward
    for n in kernels:
        assert _meta(asm["attn"], n, "vgpr_spill_count") == 0, n
        assert _meta(asm["attn"], n, "private_segment_fixed_size") == 0, n
    for name, body in _functions(asm["attn"], "_ZN4alch19k_attn_bwd_dkv_mfma"):
        for lab, txt in _blocks(body):
            if txt.count("v_mfma_") >= 16:
                assert "scratch_" not in txt, (name, lab)
