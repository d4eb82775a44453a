"""CPU-only checks of the C-ABI boundary: the built library loads without a GPU, exports every function the
public header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2406_18200_amd as sv
from paper_2406_18200_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sv.library_path()):
        from paper_2406_18200_amd.build import build
        build(verbose=False)
    return sv.load_library()


def _declared_functions():
    import glob
    text = "".join(open(h).read() for h in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(seed_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert {"seed_verify_init", "seed_verify_step", "seed_draft_step", "seed_accept_resample"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(B.EXPORTS) == set(names)


def test_workspace_size_and_config_validation(lib):
    ok = B.ModelShape(2, 256, 4, 64, 1024, 1024, "fp32").to_c()
    assert lib.seed_verify_workspace_bytes(C.byref(ok)) > 0
    big = B.ModelShape(32, 4096, 32, 128, 11008, 32000, "bf16", max_branches=16, max_rows_per_branch=6,
                       max_shared=2048, max_private=128).to_c()
    n = lib.seed_verify_workspace_bytes(C.byref(big))
    assert 13.2e9 < n < 20e9            # packed 7B weights + caches + scratch
    for kw, code in ((dict(head_dim=96), -2), (dict(d_model=4100), -2), (dict(dtype_code=7), -5),
                     (dict(max_branches=100, max_rows_per_branch=8), -3), (dict(n_layers=0), -1)):
        c = B.ModelShape(32, 4096, 32, 128, 11008, 32000, "bf16").to_c()
        for k, v in kw.items():
            setattr(c, "dtype" if k == "dtype_code" else k, v)
        assert lib.seed_verify_workspace_bytes(C.byref(c)) == 0
        h = C.c_void_p()
        rc = lib.seed_verify_init(C.byref(h), C.byref(c), None, None, 0, None)
        assert rc == code, (kw, rc, lib.seed_last_error())
        assert lib.seed_last_error()
    assert lib.seed_verify_workspace_bytes(None) == 0


def test_init_rejects_null_and_small_workspace_without_a_gpu(lib):
    c = B.ModelShape(2, 256, 4, 64, 1024, 1024, "fp32").to_c()
    h = C.c_void_p()
    assert lib.seed_verify_init(None, C.byref(c), None, None, 0, None) == -4
    assert lib.seed_verify_init(C.byref(h), C.byref(c), None, None, 0, None) == -4
    assert h.value is None


def test_stateless_entry_points_validate_arguments(lib):
    a = B.AcceptArgsC()
    a.n_branches, a.gamma, a.n_target_rows, a.vocab = 2, 3, 5, 100
    assert lib.seed_accept_resample(C.byref(a), None) == -2          # rows must be gamma or gamma + 1
    a.n_target_rows = 3
    assert lib.seed_accept_resample(C.byref(a), None) == -4          # NULL arrays
    a.n_branches = 0
    assert lib.seed_accept_resample(C.byref(a), None) == 0           # empty batch: nothing to do
    assert lib.seed_accept_resample(None, None) == -4
    assert lib.seed_sample_probs(None, 10, None, None, 0, 10, None) == 0
    assert lib.seed_sample_probs(None, 10, None, None, 3, 10, None) == -4
    assert lib.seed_sample_probs(None, 5, None, None, 3, 10, None) == -1
    for fn in (lib.seed_verify_step, lib.seed_draft_step):
        assert fn(None, None) == -6                                   # no context
    assert lib.seed_kv_load(None, 0, None, None, 0, None, None, 0, 0) == -6
    assert lib.seed_verify_status(None, None) == -6
    lib.seed_verify_destroy(None)                                     # no-op


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    """There is no CPU fallback: a missing shared library is an error, not a silent detour."""
    monkeypatch.setattr(B, "_LIB", None)
    monkeypatch.setattr(B, "HERE", str(tmp_path))
    with pytest.raises(RuntimeError, match="missing"):
        B.load_library()


def test_scheduler_argument_validation_without_a_gpu(lib):
    """seed_sched_run / seed_sched_workspace_bytes reject bad arguments before touching the GPU."""
    assert lib.seed_sched_workspace_bytes(0, 4, 32000) == 0
    assert lib.seed_sched_workspace_bytes(3, 0, 32000) == 0
    assert lib.seed_sched_workspace_bytes(64, 4, 32000) == 0          # more than SEED_SCHED_MAX_BRANCHES
    n = lib.seed_sched_workspace_bytes(3, 4, 32000)
    assert n >= 3 * 3 * 4 * 32000 * 4                                   # q rows of the units in flight
    a = B.SchedArgsC()
    assert lib.seed_sched_run(None, None, C.byref(a)) == -6             # SEED_E_NOT_INIT
    assert b"context" in lib.seed_last_error()
