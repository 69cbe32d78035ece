"""Batches larger than one pass of the workspace: the forward then runs in chunks of whole 64-state tiles.

The bf16 IMPALA teacher needs about 165 KB of workspace per state, so its configured batch of 16384 runs as three
passes; a child process repeats a student forward with the pass size forced down to 1024 states (override 1040,
rounded down to whole tiles) at B = 4133, which must give the bits of the single-pass run."""
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import policies, rel_err_rows, student_tensors, teacher_tensors, check_actions, check_sampler_self_consistency

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_bf16_teacher_config3_full_batch_crosses_chunks():
    import paper_2211_15023_amd as A
    A.load_library()
    nt, pt, ns, ps, qp = policies(3)
    B = 16384
    pol = A.Policy(nt, "bf16", teacher_tensors(pt))
    plan = A.accerl_plan_describe(pol.arch, A.pack_weights(teacher_tensors(pt)))
    chunk = int(plan.split("chunk=")[1].split()[0])
    assert 0 < chunk < B and chunk % 64 == 0, plan.splitlines()[0]
    print(f"config 3 bf16 teacher B={B}, passes of {chunk} states: generating frames", flush=True)
    x = wl.make_frames_u8(B)
    u = wl.make_uniforms(B)
    logits, value, action = pol.forward(dev(x), dev(u))
    torch.cuda.synchronize()
    # rows on both sides of every pass boundary, the batch edges, and a seeded sample
    rows = set(range(16)) | set(range(B - 16, B))
    for c0 in range(chunk, B, chunk):
        rows |= set(range(c0 - 16, c0 + 16))
    rows |= set(np.random.default_rng(3).choice(B, 32, replace=False).tolist())
    rows = np.array(sorted(rows))
    print(f"  oracle on {len(rows)} rows", flush=True)
    ref = oracle.forward_float(nt, pt, x[rows], u[rows], "bf16")
    gl, gv, ga = logits.cpu().numpy(), value.cpu().numpy(), action.cpu().numpy()
    assert rel_err_rows(gl[rows], ref["logits"]).max() <= 2e-2
    assert rel_err_rows(gv[rows], ref["value"]).max() <= 2e-2
    check_actions(ga[rows], ref["action"], ref["logits"], u[rows], 2e-2)
    check_sampler_self_consistency(ga, gl, u)
    pol.close()


CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import numpy as np, torch
import workloads as wl
import paper_2211_15023_amd as A
from helpers import policies, student_tensors
A.load_library()
nt, pt, ns, ps, qp = policies({ci})
x = wl.make_frames_u8({B}); u = wl.make_uniforms({B})
pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
plan = A.accerl_plan_describe(pol.arch, A.pack_weights(student_tensors(qp)), A.pack_scales(qp.act_scales, student_tensors(qp)))
assert "chunk=1024" in plan.splitlines()[0], plan.splitlines()[0]
logits, value, action = pol.forward(torch.from_numpy(x).cuda(), torch.from_numpy(u).cuda())
torch.cuda.synchronize()
np.savez({out!r}, logits=logits.cpu().numpy(), value=value.cpu().numpy(), action=action.cpu().numpy())
"""


@pytest.mark.parametrize("ci,B", [(2, 4133), (3, 2100)])
def test_student_in_small_passes_is_bit_identical(tmp_path, ci, B):
    import paper_2211_15023_amd as A
    A.load_library()
    out = str(tmp_path / "child.npz")
    print(f"child process: cfg{ci} B={B} in passes of 1024 states", flush=True)
    r = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), ci=ci, B=B, out=out)],
                       env=dict(os.environ, ACCERL_CHUNK="1040"), capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, r.stderr[-2000:]
    got = np.load(out)
    nt, pt, ns, ps, qp = policies(ci)
    x = wl.make_frames_u8(B)
    u = wl.make_uniforms(B)
    pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
    logits, value, action = pol.forward(dev(x), dev(u))
    torch.cuda.synchronize()
    pol.close()
    assert np.array_equal(logits.cpu().numpy(), got["logits"])
    assert np.array_equal(value.cpu().numpy(), got["value"])
    assert np.array_equal(action.cpu().numpy(), got["action"])
    rows = np.r_[0:32, 1008:1040, 2032:2064, B - 32:B]
    ref = oracle.forward_int8(ns, qp, x[rows], u[rows])
    assert np.array_equal(got["logits"][rows], ref["logits"]) and np.array_equal(got["value"][rows], ref["value"])
    check_actions(got["action"][rows], ref["action"], ref["logits"], u[rows], 1e-5)
