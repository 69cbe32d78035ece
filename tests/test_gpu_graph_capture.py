"""The forward call enqueues kernels only (no allocation, no memset, no synchronisation once the policy has run at a
batch size), so a caller may capture it into a HIP graph.  Captured once, replayed several times with eager work and
synchronisations in between and new inputs written into the same buffers, every replay must give the bits of an
eager call on the same inputs.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from helpers import policies, student_tensors

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("ci,B", [(2, 160), (1, 1024), (3, 21)])
def test_forward_replays_from_a_graph(ci, B):
    import paper_2211_15023_amd as A
    A.load_library()
    nt, pt, ns, ps, qp = policies(ci)
    pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)

    def states(first):
        if ns.obs_dtype == "u8":
            return wl.make_frames_u8(B, *ns.obs_shape, first=first)
        return wl.make_obs_f32(B, ns.obs_shape[0], first=first)

    x = torch.from_numpy(states(0)).cuda()
    u = torch.from_numpy(wl.make_uniforms(B)).cuda()
    outs = pol.alloc_outputs(B)
    eager_outs = pol.alloc_outputs(B)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        pol.forward(x, u, outputs=outs, stream=s)          # first call at this batch size: workspace, kernel attributes
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        print(f"capture cfg{ci} B={B}", flush=True)
        with torch.cuda.graph(g, stream=s):
            pol.forward(x, u, outputs=outs, stream=s)
    torch.cuda.synchronize()
    for rep in range(4):
        x.copy_(torch.from_numpy(states(1000 * rep + 7)))   # new inputs in the captured buffers
        u.copy_(torch.from_numpy(wl.make_uniforms(B, first=1000 * rep + 7)))
        for o in outs:
            o.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        pol.forward(x, u, outputs=eager_outs)               # eager work between the replays
        torch.cuda.synchronize()
        for a, b in zip(outs, eager_outs):
            assert torch.equal(a, b), (ci, B, rep)
    pol.close()
