"""Parity at the full benchmark sizes, in the launch configuration bench.py times.

The whole batch goes through the HIP path; the oracle recomputes a sample of rows (the first and last
128, which sit on tile and chunk edges, plus a seeded stride sample in between) one by one -- states are
independent rows, so a sampled row is checked exactly as in the small-batch tests.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import policies, rel_err_rows, student_tensors, teacher_tensors, check_actions, check_sampler_self_consistency

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2211_15023_amd as A
    A.load_library()
    return A


def sample_rows(B, n_mid, seed):
    edge = min(128, B // 2)
    rows = set(range(edge)) | set(range(B - edge, B))
    rng = np.random.default_rng(seed)
    rows |= set(rng.choice(B, size=min(n_mid, B), replace=False).tolist())
    return np.array(sorted(rows))


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# 4133: the large-batch kernels with a last workgroup of 37 states (two whole tiles of 16 and a cut one)
@pytest.mark.parametrize("ci,B,n_mid", [(2, 4096, 512), (2, 4133, 128), (3, 1024, 128), (3, 16384, 64)])
def test_cnn_student_full_batch_sampled(A, ci, B, n_mid):
    nt, pt, ns, ps, qp = policies(ci)
    print(f"full-size student cfg{ci} B={B}: generating frames", flush=True)
    x = wl.make_frames_u8(B)
    u = wl.make_uniforms(B)
    pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
    print("  forward", flush=True)
    logits, value, action = pol.forward(dev(x), dev(u))
    torch.cuda.synchronize()
    rows = sample_rows(B, n_mid, ci * 1000 + B)
    print(f"  oracle on {len(rows)} rows", flush=True)
    ref = oracle.forward_int8(ns, qp, x[rows], u[rows])
    assert np.array_equal(logits.cpu().numpy()[rows], ref["logits"])
    assert np.array_equal(value.cpu().numpy()[rows], ref["value"])
    check_actions(action.cpu().numpy()[rows], ref["action"], ref["logits"], u[rows], 1e-5)
    # properties that hold for every row
    a = action.cpu().numpy()
    assert a.min() >= 0 and a.max() < ns.n_actions and np.isfinite(logits.cpu().numpy()).all()
    pol.close()


def test_cnn_teacher_full_batch_sampled(A):
    nt, pt, ns, ps, qp = policies(2)
    B = 4096
    x = wl.make_frames_u8(B)
    u = wl.make_uniforms(B)
    pol = A.Policy(nt, "bf16", teacher_tensors(pt))
    logits, value, action = pol.forward(dev(x), dev(u))
    torch.cuda.synchronize()
    rows = sample_rows(B, 128, 77)
    ref = oracle.forward_float(nt, pt, x[rows], u[rows], "bf16")
    assert rel_err_rows(logits.cpu().numpy()[rows], ref["logits"]).max() <= 2e-2
    assert rel_err_rows(value.cpu().numpy()[rows], ref["value"]).max() <= 2e-2
    check_actions(action.cpu().numpy()[rows], ref["action"], ref["logits"], u[rows], 2e-2)
    check_sampler_self_consistency(action.cpu().numpy(), logits.cpu().numpy(), u)      # every row
    pol.close()


def test_recurrent_student_full_batch_sampled(A):
    """Config 4 at its batch of 4096: one environment step with done flags, sampled rows."""
    nt, pt, ns, ps, qp = policies(4)
    B = 4096
    x = wl.make_frames_u8(B)
    u = wl.make_uniforms(B)
    h0, c0 = wl.make_hc(B, 256)
    done = wl.make_done(16, B)[3]
    pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
    dh, dc = dev(h0), dev(c0)
    logits, value, action = pol.forward(dev(x), dev(u), done=dev(done), h=dh, c=dc)
    torch.cuda.synchronize()
    rows = sample_rows(B, 64, 4)
    rows = np.union1d(rows, np.nonzero(done)[0][:16])
    ref = oracle.forward_int8(ns, qp, x[rows], u[rows], h=h0[rows], c=c0[rows], done=done[rows])
    assert rel_err_rows(logits.cpu().numpy()[rows], ref["logits"]).max() <= 2e-3
    assert np.abs(dh.cpu().numpy()[rows] - ref["h"]).max() <= 1e-4 * max(1.0, np.abs(ref["h"]).max())
    assert np.abs(dc.cpu().numpy()[rows] - ref["c"]).max() <= 1e-4 * max(1.0, np.abs(ref["c"]).max())
    check_actions(action.cpu().numpy()[rows], ref["action"], ref["logits"], u[rows], 2e-3)
    pol.close()


def test_single_state_and_odd_batches(A):
    """B = 1 and batches that end inside a pixel tile, an image batch and a GEMM tile."""
    nt, pt, ns, ps, qp = policies(2)
    pol = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
    # 513 and 1030: more pairs / groups of four than resident workgroups, an odd tail, a last tile of 16 states cut short
    for B in (1, 2, 7, 65, 129, 513, 1030):
        x = wl.make_frames_u8(B, first=500)
        u = wl.make_uniforms(B, first=500)
        ref = oracle.forward_int8(ns, qp, x, u)
        logits, value, action = pol.forward(dev(x), dev(u))
        torch.cuda.synchronize()
        assert np.array_equal(logits.cpu().numpy(), ref["logits"]), B
        assert np.array_equal(value.cpu().numpy(), ref["value"]), B
        check_actions(action.cpu().numpy(), ref["action"], ref["logits"], u, 1e-5)
    pol.close()
