"""The specialised kernels against the generic ones, and the two requantization forms, on whole forwards.

The planner picks the pipelined conv1+conv2 kernel, the third-convolution kernel, the fragment-order handoff and
the streaming dense kernel for the paper's original network, and the three-instruction requantization where the
accumulators provably stay below 2^23, and for the IMPALA student whole stacks in one kernel; environment switches,
read when the library first plans or launches, select the generic kernels, the four-instruction form, or switch single
planner decisions off.  A child process runs with the switches set and hands its
outputs back through a file; both processes must produce the same bits, and the child's are checked against the
oracle on the rows it recomputes.
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

GENERIC = dict(ACCERL_NO_CONV_FRONT="1", ACCERL_NO_CONV_TAIL="1", ACCERL_NO_GEMM_STREAM="1", ACCERL_NO_FRAG_HANDOFF="1")
PLAIN_REQUANT = dict(ACCERL_NO_P23="1")

CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import numpy as np, torch
import workloads as wl
import paper_2211_15023_amd as A
from helpers import policies, student_tensors, teacher_tensors
A.load_library()
nt, pt, ns, ps, qp = policies({ci})
x = wl.make_frames_u8({B}); u = wl.make_uniforms({B})
if {role!r} == "student":
    pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
else:
    pol = A.Policy(nt, "bf16", teacher_tensors(pt))
logits, value, action = pol.forward(torch.from_numpy(x).cuda(), torch.from_numpy(u).cuda())
torch.cuda.synchronize()
np.savez({out!r}, logits=logits.cpu().numpy(), value=value.cpu().numpy(), action=action.cpu().numpy())
"""

CASES = [
    # 4133 states of config 2: the large-batch kernels, with a last workgroup of 37 states
    ("generic", GENERIC, 2, 4133, "student"),
    ("plain-requant", PLAIN_REQUANT, 2, 4133, "student"),
    # 23 states of config 3: the stack and residual-block kernels with their last batches cut short
    ("plain-requant", PLAIN_REQUANT, 3, 23, "student"),
    # the planner decisions of the IMPALA student one by one: whole stacks -> single blocks -> layer by layer,
    # pooling as a kernel of its own, thin layers without pixel packing / without their small batches
    ("no-stack", dict(ACCERL_NO_STACK_FUSE="1"), 3, 23, "student"),
    ("no-resblock", dict(ACCERL_NO_RESBLOCK_FUSE="1"), 3, 23, "student"),
    ("no-pool-fuse", dict(ACCERL_NO_POOL_FUSE="1"), 3, 23, "student"),
    ("no-pixel-pack", dict(ACCERL_NO_PIXEL_PACK="1"), 3, 23, "student"),
    ("no-thin", dict(ACCERL_NO_THIN="1"), 3, 23, "student"),
    # config 2 through the generic convolution kernels, without the wave-private variant / without fusing conv1 + conv2
    ("no-wave-private", dict(ACCERL_NO_CONV_FRONT="1", ACCERL_NO_CONV_TAIL="1", ACCERL_NO_WAVE_PRIVATE="1"), 2, 77, "student"),
    ("no-conv-fuse", dict(ACCERL_NO_CONV_FRONT="1", ACCERL_NO_CONV_FUSE="1"), 2, 77, "student"),
    # bf16 teacher with the observation bytes converted through the 256-entry table instead of in registers
    ("obs-table", dict(ACCERL_OBS_LUT="1"), 2, 37, "teacher"),
]


@pytest.mark.parametrize("name,env,ci,B,role", CASES, ids=[f"{c[0]}-cfg{c[2]}-B{c[3]}" for c in CASES])
def test_kernel_choices_agree(tmp_path, name, env, ci, B, role):
    import paper_2211_15023_amd as A
    from helpers import teacher_tensors, rel_err_rows
    A.load_library()
    out = str(tmp_path / "child.npz")
    print(f"child process: {name}, cfg{ci} B={B} {role}", flush=True)
    r = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), ci=ci, B=B, out=out, role=role)],
                       env=dict(os.environ, **env), capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, r.stderr[-2000:]
    gen = np.load(out)

    nt, pt, ns, ps, qp = policies(ci)
    x = wl.make_frames_u8(B)
    u = wl.make_uniforms(B)
    pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales) if role == "student" else A.Policy(nt, "bf16", teacher_tensors(pt))
    print("this process: default plan", flush=True)
    logits, value, action = pol.forward(torch.from_numpy(x).cuda(), torch.from_numpy(u).cuda())
    torch.cuda.synchronize()
    pol.close()
    # both plans compute the same bits (also the bf16 teacher: same values staged, same kernels behind them)
    assert np.array_equal(logits.cpu().numpy(), gen["logits"])
    assert np.array_equal(value.cpu().numpy(), gen["value"])
    assert np.array_equal(action.cpu().numpy(), gen["action"])
    rows = np.r_[0:min(64, B // 2), B - min(64, B // 2):B]
    if role == "student":
        ref = oracle.forward_int8(ns, qp, x[rows], u[rows])
        assert np.array_equal(gen["logits"][rows], ref["logits"])
        assert np.array_equal(gen["value"][rows], ref["value"])
        check_actions(gen["action"][rows], ref["action"], ref["logits"], u[rows], 1e-5)
    else:
        ref = oracle.forward_float(nt, pt, x[rows], u[rows], "bf16")
        assert rel_err_rows(gen["logits"][rows], ref["logits"]).max() <= 2e-2
        check_actions(gen["action"][rows], ref["action"], ref["logits"], u[rows], 2e-2)
