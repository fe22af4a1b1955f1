"""The forward and backward calls only enqueue kernels (no allocation, synchronisation or memset),
so a caller may record them into a HIP graph.  Replays are checked against the eager results,
with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

import gen
from helpers import Problem, to_torch

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("lean", [False, True])
def test_forward_backward_under_graph_capture(lean):
    import paper_2604_16715_amd as gta
    p = Problem.from_workload(gen.workload("mid", 8))
    print(f"graph-capture case lean={lean} nnz={int(p.indptr[-1])}", flush=True)
    plan = gta.gta_plan_create(torch.from_numpy(p.indptr).cuda(), torch.from_numpy(p.indices).cuda(), p.n_src,
                               wave_max_deg=16, hub_chunk=64, keep_dz_min_nnz=1)
    Q, K, V, dO = (to_torch(getattr(p, k)) for k in ("Q", "K", "V", "dO"))
    out, lse = torch.empty_like(Q), torch.empty((p.n_dst, Q.shape[1]), dtype=torch.float32, device="cuda")
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)

    def step():
        gta.gta_attn_fwd(plan, Q, K, V, 0.0, out, lse)
        gta.gta_attn_bwd(plan, Q, K, V, out, lse, dO, 0.0, dQ, dK, dV, lean_scratch=lean)

    step()   # eager reference (also allocates the scratch buffers before capture)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (out, lse, dQ, dK, dV)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        for t in (out, lse, dQ, dK, dV):
            t.fill_(float("nan") if t.is_floating_point() else 0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((out, lse, dQ, dK, dV), ref):
            assert torch.equal(got, want), f"replay {rep} differs from the eager result"
        # eager work between replays
        step()
        torch.cuda.synchronize()
