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


@pytest.mark.parametrize("N,gamma,S,R", [(3, 4, 100, 0), (5, 3, 70, 9), (16, 6, 257, 40), (1, 1, 33, 0),
                                         (2, 5, 1100, 300),   # <= 16 rows, 13 partials: in-launch merge in passes
                                         (1, 40, 64, 20),     # one branch of 40 rows: two row groups per branch
                                         (3, 7, 200, 150)])   # 21 rows (two row tiles), two private key ranges
def test_small_bf16_synthetic_kv(N, gamma, S, R):
    """Small bf16 model (2 layers, d=256, 4 heads of 64): several MFMA tiles, ragged tails in rows and keys,
    and every shape of the attention launch (one / two row tiles, merge inside / after the launch, several
    key ranges in the shared and the private segment, several row groups per branch)."""
    w = wl.get_workload("c3").scaled(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ff=704, vocab=2000,
                                     N=N, gamma=gamma, S=S, R=R, seed=77 + N)
    Case(w).run_oracle().run_gpu().compare()


def test_small_bf16_head128_long_private_context():
    """head_dim 128, 12 rows against 1000 shared and 260 private keys (three private key ranges)."""
    w = wl.get_workload("c3").scaled(n_layers=2, d_model=512, n_heads=4, head_dim=128, d_ff=1024, vocab=4096,
                                     N=3, gamma=4, S=1000, R=260, seed=93)
    Case(w).run_oracle().run_gpu().compare()


def test_small_bf16_true_prefix_head128():
    w = wl.get_workload("c2").scaled(n_layers=2, d_model=512, n_heads=4, head_dim=128, d_ff=1024, vocab=4096,
                                     N=6, gamma=5, S=150, R=11, seed=91)
    Case(w).run_oracle().run_gpu().compare()


def test_perturbed_draft_q_13b_widths_two_layers():
    """13B widths (d=5120, 40 heads, F=13824) at two layers, N=8 x gamma=5, S=4096, with the draft
    distribution a perturbed copy of the target's, built autoregressively by the oracle: realistic
    acceptance rates, so the accept / resample path sees both outcomes."""
    import harness
    w = wl.get_workload("c5").scaled(n_layers=2)
    W = harness.CachedWeights(wl.Weights(w.model, w.seed))
    q = harness.perturbed_q_autoregressive(w, W)
    c = Case(w, q_override=q).run_oracle().run_gpu()
    c.compare()
    assert 0 < c.ref_accept[0].sum() < w.N * w.gamma


def test_results_are_bit_identical_from_run_to_run():
    """No floating-point atomics anywhere: the same step twice gives the same bits (split-K partials are
    summed by the last workgroup in a fixed order)."""
    import torch
    w = wl.get_workload("c3").scaled(n_layers=2, N=16, gamma=6, S=300, R=17)
    c = Case(w).run_oracle().run_gpu(keep_ctx=True)
    first = (c.gpu_logits.copy(), [a.copy() for a in c.gpu_accept])
    for _ in range(3):
        c.dev_plen.fill_(w.R)
        c.dev_logits.zero_()
        import workloads.device as D
        inp = c.inp
        acc = dict(q=D.f32(inp["q"]), draft_tok=D.i32(inp["drafts"]), u_acc=D.f32(inp["u_acc"]), u_res=D.f32(inp["u_res"]),
                   temperature=w.temperature)
        outs = c.ctx.step(D.i32(inp["row_tok"]), w.S, c.dev_plen, logits_out=c.dev_logits, accept=acc)
        torch.cuda.synchronize()
        assert np.array_equal(c.dev_logits.cpu().numpy(), first[0])
        for a, b in zip(outs, first[1]):
            assert np.array_equal(a.cpu().numpy(), b)
    c.ctx.close()


def test_private_capacity_overflow_is_flagged_not_fatal():
    import torch
    import workloads.device as D
    w = wl.get_workload("c1").scaled(N=2, gamma=3)
    c = Case(w).run_oracle().run_gpu(keep_ctx=True)       # max_private = 0: one step fits exactly
    assert c.status == 0
    inp = c.inp
    acc = dict(q=D.f32(inp["q"]), draft_tok=D.i32(inp["drafts"]), u_acc=D.f32(inp["u_acc"]), u_res=D.f32(inp["u_res"]),
               temperature=w.temperature)
    c.ctx.step(D.i32(inp["row_tok"]), w.S, c.dev_plen, accept=acc)     # private_len is now >= 1 > max_private
    torch.cuda.synchronize()
    assert c.ctx.status() & 1
    assert c.ctx.status() == 0                                          # reading clears the word
    c.ctx.close()


def test_empty_and_single_row_steps():
    import torch
    import workloads.device as D
    w = wl.get_workload("c1")
    c = Case(w).run_oracle().run_gpu(keep_ctx=True)
    empty = torch.zeros((0, 4), dtype=torch.int32, device="cuda")
    assert c.ctx.step(empty, w.S, c.dev_plen) is None                   # N = 0: nothing launched, no error
    c.ctx.close()
    Case(w.scaled(N=1, gamma=1)).run_oracle().run_gpu().compare()
