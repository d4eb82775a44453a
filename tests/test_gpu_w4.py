"""GPU parity of the four-bit-weight mode (context dtype "bf16w4": projection matrices streamed as MXFP4 -- E2M1
codes with one power-of-two scale per 32 inputs -- a quarter of the bytes of the bf16 weight stream) through the C
ABI.  As for the one-byte mode the oracle is unchanged: it is handed the dequantised weights, i.e. exactly the values
the codes and scales stand for, so the bf16-path tolerance applies; the error against the UNQUANTISED weights is a
property of the format, printed for the record."""
import numpy as np
import pytest

import workloads as wl
from harness import Case

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,gamma,S,R,bonus", [(3, 4, 100, 0, False), (8, 5, 257, 40, False), (16, 6, 300, 17, False),
                                               (5, 3, 70, 9, True), (1, 1, 33, 0, False)])
def test_small_w4_synthetic_kv(N, gamma, S, R, bonus):
    """12, 40, 96, 20 and 1 rows (one, three and 2 x three row tiles: the row-share launches included)."""
    w = wl.get_workload("c3").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000, N=N,
                                     gamma=gamma, S=S, R=R, seed=977 + N, dtype="bf16w4")
    Case(w, bonus=bonus).run_oracle().run_gpu().compare()


def test_w4_wide_shapes_ragged_k_and_many_rows():
    """Outputs of 600 and 1300 n-tiles with a k extent of 18 k-tiles at 96, 40 and 250 rows."""
    for N, gamma in ((16, 6), (8, 5), (50, 5)):
        w = wl.get_workload("c4").scaled(n_layers=2, d_model=576, n_heads=9, head_dim=64, d_ff=4800, vocab=20800, N=N,
                                         gamma=gamma, S=100, R=20, seed=1077 + gamma, dtype="bf16w4")
        Case(w, branches=[0, N // 2, N - 1]).run_oracle().run_gpu().compare()


def test_w4_13b_widths_two_layers_and_error_of_the_format():
    """13B widths (d = 5120, F = 13824) at two layers, N = 8 x gamma = 5 over 4096 shared tokens.  Also prints how
    far the four-bit weights move the logits away from those of the bf16 weights they were made from."""
    w = wl.get_workload("c5").scaled(n_layers=2, q_kind="random", q_temp=1.0, dtype="bf16w4")
    c = Case(w, branches=[0, 5]).run_oracle().run_gpu()
    c.compare()
    wb = w.scaled(dtype="bf16")
    cb = Case(wb, branches=[0, 5]).run_oracle()
    d = c.gpu_logits[[0, 5]] - cb.ref_logits
    print(f"four-bit weights vs the bf16 weights (2 layers, 13B widths): rms logit difference {np.sqrt((d * d).mean()):.4f}, "
          f"max {np.abs(d).max():.4f}, rms logit {np.sqrt((cb.ref_logits ** 2).mean()):.4f}", flush=True)
    assert np.sqrt((d * d).mean()) < 0.8 * np.sqrt((cb.ref_logits ** 2).mean())
