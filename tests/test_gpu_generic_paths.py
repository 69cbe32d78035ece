"""The specialised kernels of the paper's original network against the generic ones on whole forwards.

The planner picks the pipelined conv1+conv2 kernel, the third-convolution kernel, the fragment-order handoff and
the streaming dense kernel for this network; environment switches, read when the library first plans or launches,
send the same network through the generic convolution and dense kernels instead.  A child process runs with the
switches set and hands its outputs back through a file; both processes must produce the same bits, and both are
checked against the oracle on the rows it recomputes.
"""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import policies, student_tensors, check_actions

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
B = 4133           # large-batch kernels, with a last workgroup of 37 states

CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import numpy as np, torch
import workloads as wl
import paper_2211_15023_amd as A
from helpers import policies, student_tensors
A.load_library()
nt, pt, ns, ps, qp = policies(2)
x = wl.make_frames_u8({B}); u = wl.make_uniforms({B})
pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
logits, value, action = pol.forward(torch.from_numpy(x).cuda(), torch.from_numpy(u).cuda())
torch.cuda.synchronize()
np.savez({out!r}, logits=logits.cpu().numpy(), value=value.cpu().numpy(), action=action.cpu().numpy())
"""


def test_generic_and_specialised_kernels_agree(tmp_path):
    import paper_2211_15023_amd as A
    A.load_library()
    out = str(tmp_path / "generic.npz")
    env = dict(os.environ, ACCERL_NO_CONV_FRONT="1", ACCERL_NO_CONV_TAIL="1", ACCERL_NO_GEMM_STREAM="1",
               ACCERL_NO_FRAG_HANDOFF="1")
    print("child process: generic kernels", flush=True)
    r = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), B=B, out=out)],
                       env=env, capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, r.stderr[-2000:]
    gen = np.load(out)

    nt, pt, ns, ps, qp = policies(2)
    x = wl.make_frames_u8(B)
    u = wl.make_uniforms(B)
    pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
    print("this process: specialised kernels", flush=True)
    logits, value, action = pol.forward(torch.from_numpy(x).cuda(), torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    pol.close()
    assert np.array_equal(logits.cpu().numpy(), gen["logits"])
    assert np.array_equal(value.cpu().numpy(), gen["value"])
    assert np.array_equal(action.cpu().numpy(), gen["action"])
    rows = np.r_[0:64, B - 64:B]
    ref = oracle.forward_int8(ns, qp, x[rows], u[rows])
    assert np.array_equal(gen["logits"][rows], ref["logits"])
    assert np.array_equal(gen["value"][rows], ref["value"])
    check_actions(gen["action"][rows], ref["action"], ref["logits"], u[rows], 1e-5)
