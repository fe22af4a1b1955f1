"""Head-split / head-merge layout transforms against their definition (a numpy transpose):
byte-exact."""
import numpy as np
import pytest
import torch

import gen
from helpers import to_torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,heads,head_dim,dtype,parts", [
    (1000, 8, 16, "f32", 2), (1000, 8, 16, "f32", 8), (777, 8, 32, "bf16", 4), (1, 4, 64, "bf16", 4),
    (4099, 16, 8, "bf16", 2), (300, 4, 16, "f32", 1), (0, 8, 16, "f32", 2),
])
def test_head_split_and_merge(n, heads, head_dim, dtype, parts):
    import paper_2604_16715_amd as gta
    print(f"layout case n={n} heads={heads} head_dim={head_dim} {dtype} parts={parts}", flush=True)
    x = gen.normal((max(n, 1), heads, head_dim), dtype, 11, 2)[:n]
    X = to_torch(np.ascontiguousarray(x))
    S = gta.gta_head_split(X, parts)
    # definition: block r holds heads [r*h/p, (r+1)*h/p) of every row
    want = x.reshape(n, parts, heads // parts, head_dim).transpose(1, 0, 2, 3)
    got = S.view(torch.int16 if dtype == "bf16" else torch.int32).cpu().numpy()
    np.testing.assert_array_equal(got, np.ascontiguousarray(want).view(got.dtype))
    back = gta.gta_head_merge(S)
    assert torch.equal(back.view(torch.int16 if dtype == "bf16" else torch.int32),
                       X.view(torch.int16 if dtype == "bf16" else torch.int32))


def test_head_split_rejects_bad_arguments():
    import paper_2604_16715_amd as gta
    X = torch.zeros((10, 6, 16), device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_head_split(X, 4)            # 6 heads not divisible by 4
    X = torch.zeros((10, 4, 2), device="cuda")
    with pytest.raises(gta.GtaError):
        gta.gta_head_split(X, 4)            # 8-byte head blocks
