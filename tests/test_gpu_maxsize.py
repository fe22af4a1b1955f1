"""One problem with more than 2^30 stored entries (the library's limit is 2^31): entry positions
no longer fit in 30 bits and byte offsets into the 4-byte per-entry arrays pass 2^32.  Sixteen
million-entry hub rows go through the chunk + merge schedule, a thousand rows are empty.  Checked
like the other full-size cases: the oracle computes sampled rows, identities cover the rest."""
import numpy as np
import pytest

import gen
from helpers import Problem, sampled_parity

pytestmark = pytest.mark.gpu


def test_more_than_2_pow_30_entries():
    n, heads, head_dim = 1 << 20, 4, 8          # 64-byte bf16 rows keep the tensors small
    rng = np.random.Generator(np.random.Philox(0x260416715 + 99))
    deg = rng.integers(800, 1301, size=n).astype(np.int64)
    deg[rng.choice(n, size=1000, replace=False)] = 0
    hubs = rng.choice(n, size=4, replace=False)
    deg[hubs] = 3_000_000
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=indptr[1:])
    nnz = int(indptr[-1])
    assert (1 << 30) < nnz < (1 << 31)
    print(f"max-size case: nnz={nnz}; drawing sources", flush=True)
    indices = rng.integers(0, n, size=nnz, dtype=np.int32)   # repeated sources inside a row are allowed
    p = Problem.random(indptr, indices, n, heads, head_dim, "bf16", seed=4242)
    sampled_parity(p, "max-size", 4242, nnz, dst_count=60, src_count=4)
