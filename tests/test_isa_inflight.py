"""The wide projection kernels issue their loads in inline assembly and count their own waits.  These tests
compile the kernel source to gfx950 ISA (no GPU needed) and replay every path through each kernel: no
instruction may touch a register that an outstanding load is still going to write, and no kernel may carry
spill code (scratch loads and stores would be loads in the kernel's own count)."""
import os
import subprocess
import tempfile

import pytest

from paper_2406_18200_amd import build as B
import isa_check


def test_checker_finds_a_planted_violation_and_accepts_the_fix():
    bad = """
_Zfake_kernel:
        global_load_dwordx4 v[8:11], v[0:1], off
        global_load_dwordx4 v[12:15], v[2:3], off
        s_waitcnt vmcnt(1)
        v_add_u32_e32 v20, v8, v9
        v_add_u32_e32 v21, v12, v20
        s_endpgm
.Lfunc_end0:
"""
    errs = isa_check.check_text(bad, "fake")["_Zfake_kernel"]
    assert len(errs) == 1 and "v[12:15]" in errs[0]            # the first load is covered by vmcnt(1), the second is not
    good = bad.replace("v_add_u32_e32 v21, v12, v20", "s_waitcnt vmcnt(0)\n        v_add_u32_e32 v21, v12, v20")
    assert isa_check.check_text(good, "fake")["_Zfake_kernel"] == []
    # LDS reads are counted separately, and a loop carries outstanding loads around its back edge
    loop = """
_Zfake_loop:
        ds_read_b128 v[4:7], v30
.LBB0_1:
        s_waitcnt lgkmcnt(0)
        v_mov_b32_e32 v40, v4
        ds_read_b128 v[4:7], v30 offset:1024
        s_cbranch_scc1 .LBB0_1
        v_mov_b32_e32 v41, v5
        s_endpgm
.Lfunc_end1:
"""
    errs = isa_check.check_text(loop, "fake")["_Zfake_loop"]
    assert len(errs) == 1 and "v_mov_b32_e32 v41, v5" in errs[0]


@pytest.fixture(scope="module")
def gemm_isa():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    flags = [f for f in B.FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "gemm.s")
        r = subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only", os.path.join(B.CSRC, "gemm_bf16.hip"), "-o", out],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout[-2000:]
        return open(out).read()


def test_wide_projection_kernels_touch_no_register_in_flight(gemm_isa):
    res = isa_check.check_text(gemm_isa, "gemm_wide_kernel")
    assert len(res) >= 30                                       # every instantiated shape and epilogue
    bad = {k: v[:3] for k, v in res.items() if v}
    assert not bad, bad


def test_wide_projection_kernels_have_no_spill_code(gemm_isa):
    sc = isa_check.scratch_bytes(gemm_isa, "gemm_wide_kernel")
    assert len(sc) >= 30
    assert all(v == 0 for v in sc.values()), {k: v for k, v in sc.items() if v}
