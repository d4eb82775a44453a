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
    """13B shapes, N=8 x gamma=5 over a 4096-token shared prefix, full 40 layers.  The draft distributions
    here are the random-logit kind: building the perturbed-target kind needs gamma sequential oracle passes
    over 25.7 GB of weights; that recipe is exercised at two layers in test_gpu_verify.py."""
    w = wl.get_workload("c5").scaled(q_kind="random", q_temp=1.0)
    Case(w, branches=[0, 5]).run_oracle().run_gpu().compare()


def test_c6_7b_state_evaluator_shape_sampled_branches():
    """No shared prefix, eight private contexts of 384..1024 tokens: the shortest, the longest and one between."""
    Case(wl.get_workload("c6"), branches=[0, 3, 7]).run_oracle().run_gpu().compare()
