"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (default
plan).  The oracle cannot run the whole problem in seconds, so it computes sampled output rows
one sub-problem at a time:

* a destination row's out / lse / dQ depend only on that row's entries, so the sub-problem is
  the sampled rows with all their entries (sources renumbered compactly);
* a source row's dK / dV need every entry that points to it and, for each of those, the whole
  softmax row of its destination; the sub-problem is every destination row that references a
  sampled source, with all its entries.

Two identities that hold at any size are checked on the complete GPU outputs as well.
"""
import pytest

import gen
from helpers import Problem, sampled_parity

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["large", "partition", "skew"])
def test_full_size_sampled_parity(name):
    print(f"full-size case {name}: generating", flush=True)
    w = gen.workload(name)
    sampled_parity(Problem.from_workload(w), name, w.seed, w.nnz)
