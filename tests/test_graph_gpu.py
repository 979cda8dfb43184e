"""The entry points only enqueue kernels on the stream they are given -- no allocation, no memset,
no synchronisation -- so a forward + backward pair can be captured into a HIP graph and replayed.
Each replay (with eager work and synchronisations in between, and new inputs written in place)
must reproduce the eager result bit for bit; the eager results themselves are checked against
the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from helpers import f64, max_abs, rmse
from paper_2407_08608_amd import binding, inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("noalloc", [False, True])
@pytest.mark.parametrize("causal", [False, True])
def test_forward_backward_graph_replays_match_eager(causal, noalloc):
    # noalloc: the backward on the library's own scratch (the entry point meant for callers under capture); its
    # scratch address is resolved by the eager calls below, before the capture begins
    B, H, N, d = 2, 4, 1300, 128
    scale = d ** -0.5
    sets = [tuple(t.cuda() for t in (*inputs.qkv(200 + i, B, H, N, d, "bf16"),
                                     inputs.normal_tensor(210 + i, "do", (B, H, N, d), "bf16"))) for i in range(3)]
    q, k, v, do = (torch.empty_like(t) for t in sets[0])
    o = torch.empty_like(q)
    lse = torch.empty((B, H, N), device=q.device, dtype=torch.float32)
    dq, dk, dv = (torch.empty_like(q) for _ in range(3))
    ws = torch.empty(binding.fa_bwd_workspace_bytes(B, H, N, d), device=q.device, dtype=torch.uint8)

    def step():
        binding.fa_fwd(q, k, v, scale, causal, o=o, lse=lse)
        if noalloc:
            binding.fa_bwd_noalloc(q, k, v, o, lse, do, scale, causal, dq, dk, dv)
        else:
            binding.fa_bwd(q, k, v, o, lse, do, scale, causal, dq=dq, dk=dk, dv=dv, workspace=ws)

    # eager references for the three input sets
    eager = []
    for s in sets:
        for dst, src in zip((q, k, v, do), s):
            dst.copy_(src)
        step()
        torch.cuda.synchronize()
        eager.append([t.clone() for t in (o, lse, dq, dk, dv)])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    for rep in range(2):
        for s, ref in zip(sets, eager):
            for dst, src in zip((q, k, v, do), s):
                dst.copy_(src)
            for t in (o, lse, dq, dk, dv):
                t.fill_(float("nan"))  # eager work between replays; stale results cannot pass
            graph.replay()
            torch.cuda.synchronize()
            for got, want in zip((o, lse, dq, dk, dv), ref):
                assert torch.equal(got, want), rep

    # and the eager results are right
    qc, kc, vc, doc = (f64(t) for t in sets[2])
    r = oracle.attention_bwd(qc, kc, vc, doc, scale, causal)
    o_e, l_e, dq_e, dk_e, dv_e = eager[2]
    assert max_abs(f64(o_e), r["o"]) <= 2e-2 and max_abs(f64(l_e), r["lse"]) <= 2e-3
    for got, name in ((dq_e, "dq"), (dk_e, "dk"), (dv_e, "dv")):
        ref = r[name]
        assert rmse(f64(got), ref) <= 1e-2 * float(np.sqrt(np.mean(ref * ref))) + 1e-5, name
