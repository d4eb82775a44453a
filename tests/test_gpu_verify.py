"""GPU parity of the whole verify step (forward + accept/resample) against the oracle, through the C ABI."""
import numpy as np
import pytest

import workloads as wl
from harness import Case

pytestmark = pytest.mark.gpu


def test_c1_tiny_fp32_true_prefix():
    """Tiny fp32 plumbing case: both sides compute the 64-token prefix themselves."""
    Case(wl.get_workload("c1")).run_oracle().run_gpu().compare()


def test_c1_bonus_row_and_private_context():
    w = wl.get_workload("c1").scaled(R=7, N=4)
    Case(w, bonus=True).run_oracle().run_gpu().compare()


def test_c1_greedy():
    Case(wl.get_workload("c1"), greedy=True).run_oracle().run_gpu().compare()


@pytest.mark.parametrize("N,gamma,S,R", [(3, 4, 100, 0), (5, 3, 70, 9), (16, 6, 257, 40), (1, 1, 33, 0)])
def test_small_bf16_synthetic_kv(N, gamma, S, R):
    """Small bf16 model (2 layers, d=256, 4 heads of 64): several MFMA tiles, ragged tails in rows and keys."""
    w = wl.get_workload("c3").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                     N=N, gamma=gamma, S=S, R=R, seed=77 + N)
    Case(w).run_oracle().run_gpu().compare()


def test_small_bf16_true_prefix_head128():
    w = wl.get_workload("c2").scaled(n_layers=2, d_model=512, n_heads=4, head_dim=128, d_ff=1024, vocab=4096,
                                     N=6, gamma=5, S=150, R=11, seed=91)
    Case(w).run_oracle().run_gpu().compare()
