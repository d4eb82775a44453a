"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times.  The oracle evaluates
a sample of branches (each branch's rows are independent of the other branches given the shared prefix), the
GPU runs the whole step."""
import pytest

import workloads as wl
from harness import Case

pytestmark = pytest.mark.gpu


def test_c3_7b_full_step_all_rows():
    Case(wl.get_workload("c3")).run_oracle().run_gpu().compare()


def test_c4_7b_wide_sampled_branches():
    Case(wl.get_workload("c4"), branches=[0, 7, 15]).run_oracle().run_gpu().compare()


def test_c4_7b_wide_greedy_sampled_branches():
    """The same configuration in greedy verification mode (the second mode the configuration names)."""
    Case(wl.get_workload("c4"), greedy=True, branches=[3, 12]).run_oracle().run_gpu().compare()


def test_c5_13b_sampled_branches_random_q():
    """13B shapes, N=8 x gamma=5 over a 4096-token shared prefix, full 40 layers, with the random-logit kind of
    draft distribution (two branches against the oracle in one pass)."""
    w = wl.get_workload("c5").scaled(q_kind="random", q_temp=1.0)
    Case(w, branches=[0, 5]).run_oracle().run_gpu().compare()


def test_c5_13b_as_configured_perturbed_target_q():
    """c5 exactly as configured, at full depth: the draft distribution of every position is the target's own
    distribution at that position perturbed by N(0, 0.5^2) noise on the logits (same temperature), so it
    depends on the drafts sampled before it.  For the branch that is compared, the ORACLE builds that chain
    (gamma incremental single-row passes over the 40 layers) and both sides get the same q and drafts; the other
    branches, which nothing is compared on, get theirs from the library's own single-row steps.  Slow: about
    six oracle passes over 25.7 GB of weights.  Realistic acceptance: accepted prefixes, rejections and
    replacement draws all occur at V = 32000."""
    import harness
    w = wl.get_workload("c5")
    assert w.q_kind == "perturbed" and w.model.n_layers == 40
    sel = [5]
    q = harness.perturbed_q_autoregressive(w, wl.Weights(w.model, w.seed, reuse_buffers=True), branches=sel)
    print("oracle-built draft chain ready", flush=True)
    c = Case(w, branches=sel, q_override=q).run_oracle().run_gpu()
    c.compare()
    a_all = c.gpu_accept[0]
    print("accepted per branch (library, all branches):", a_all.tolist(), flush=True)
    assert 0 < a_all.sum() < w.N * w.gamma          # both outcomes occur


def test_c6_7b_state_evaluator_shape_sampled_branches():
    """No shared prefix, eight private contexts of 384..1024 tokens: the shortest, the longest and one between."""
    Case(wl.get_workload("c6"), branches=[0, 3, 7]).run_oracle().run_gpu().compare()


def test_c8_7b_batch_sweep_768_rows_sampled_branches():
    """The largest step of the batch sweep at full size: 128 branches x 6 drafts = 768 rows on the 7B shapes, in the
    launch configuration bench.py times (row shares of the projections, 1792 attention workgroups); the first and
    the last branch against the oracle."""
    Case(wl.get_workload("c8"), branches=[0, 127]).run_oracle().run_gpu().compare()
