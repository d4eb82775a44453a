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
