"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (default
plan): the oracle runs the whole workload and every element of out, lse, dQ, dK and dV is
compared (2.4 M - 8.4 M rows, 49 M - 140 M stored entries per workload)."""
import pytest

import gen
from helpers import Problem, whole_parity

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["large", "partition", "skew"])
def test_full_size_whole_tensor_parity(name):
    print(f"whole-tensor case {name}: generating", flush=True)
    w = gen.workload(name)
    whole_parity(Problem.from_workload(w), name, w.nnz)
