"""alpha-mixture of the smaller and the original policy (Section 3.2): every row must hold exactly what
the network chosen for it produces on that row alone — int8 rows bit-exact against the oracle, bf16
rows within the bf16 tolerance, and equal to the same policy's own forward on the GPU."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import policies, make_states, rel_err_rows, student_tensors, teacher_tensors, check_actions, check_sampler_self_consistency

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2211_15023_amd as A
    A.load_library()
    return A


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("B,alpha", [(64, 0.5), (37, 0.3), (160, 0.9), (33, 0.0), (33, 1.0), (5, 0.5)])
def test_mixture_rows_match_their_network(A, B, alpha):
    # smaller = the paper's Net3 quantized to int8; original = the paper's conv 32/64/64 network in bf16
    small = wl.configs.PAPER_STUDENTS["net3"]
    ps = wl.init_params(small, wl.STREAM["weights_student"])
    qp = oracle.quantize_policy(small, ps, make_states(small, 64, wl.STREAM["calibration"]))
    orig = wl.nature_cnn()
    po = wl.init_params(orig, wl.STREAM["weights_teacher"])
    p_small = A.Policy(small, "int8", qp.tensors, qp.act_scales)
    p_orig = A.Policy(orig, "bf16", teacher_tensors(po))
    x = make_states(small, B, wl.STREAM["states"])
    u = wl.make_uniforms(B)
    use = (wl.uniform01(wl.BASE_SEED, 41, 0, B) < np.float32(alpha)).astype(np.uint8)   # Bernoulli(alpha) per row
    print(f"mixture B={B} alpha={alpha} smaller rows={int(use.sum())}", flush=True)
    ref = oracle.forward_mixture(small, qp, orig, po, "bf16", x, u, use)
    nA = small.n_actions
    logits = torch.full((B, nA), float("nan"), dtype=torch.float32, device="cuda")
    value = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
    action = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    dx, du = _dev(x), _dev(u)
    A.accerl_actor_forward_mixture(p_small.handle, p_orig.handle, dx, du, use, logits, value, action)
    torch.cuda.synchronize()
    gl, gv, ga = logits.cpu().numpy(), value.cpu().numpy(), action.cpu().numpy()
    m = use.astype(bool)
    assert np.array_equal(gl[m], ref["logits"][m]) and np.array_equal(gv[m], ref["value"][m])
    if m.any():
        check_actions(ga[m], ref["action"][m], ref["logits"][m], u[m], 1e-5)
    if (~m).any():
        assert rel_err_rows(gl[~m], ref["logits"][~m]).max() <= 2e-2
        assert rel_err_rows(gv[~m], ref["value"][~m]).max() <= 2e-2
        check_actions(ga[~m], ref["action"][~m], ref["logits"][~m], u[~m], 2e-2)
    check_sampler_self_consistency(ga, gl, u)      # every row, whichever network produced it
    # and bit-identical to what each policy computes for those rows in a plain forward
    ls, vs, as_ = p_small.forward(dx, du)
    lo, vo, ao = p_orig.forward(dx, du)
    torch.cuda.synchronize()
    tm = torch.from_numpy(m).cuda()
    assert torch.equal(logits[tm], ls[tm]) and torch.equal(action[tm], as_[tm]) and torch.equal(value[tm], vs[tm])
    assert torch.equal(logits[~tm], lo[~tm]) and torch.equal(action[~tm], ao[~tm]) and torch.equal(value[~tm], vo[~tm])
    # a second call with another draw reuses the buffers
    use2 = 1 - use
    A.accerl_actor_forward_mixture(p_small.handle, p_orig.handle, dx, du, use2, logits, value, action)
    torch.cuda.synchronize()
    tm2 = ~tm
    assert torch.equal(logits[tm2], ls[tm2]) and torch.equal(logits[~tm2], lo[~tm2])
    p_small.close(); p_orig.close()


def test_mixture_alpha_schedule(A):
    from oracle import layers as L
    for k in (0.0, 0.1, 0.2, 0.3, 0.45, 0.5, 2.0):
        assert A.accerl_mixture_alpha(k, 0.1, 0.5) == L.mixture_alpha(k, 0.1, 0.5)


def test_mixture_rejects_mismatched_policies(A):
    nt, pt, ns, ps, qp = policies(0)
    mlp = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
    small = wl.configs.PAPER_STUDENTS["net3"]
    p3 = A.Policy(small, "bf16", teacher_tensors(wl.init_params(small, wl.STREAM["weights_student"])))
    x = _dev(make_states(small, 4, wl.STREAM["states"]))
    u = _dev(wl.make_uniforms(4))
    lg = torch.empty(4, 18, device="cuda"); v = torch.empty(4, device="cuda"); a = torch.empty(4, dtype=torch.int32, device="cuda")
    with pytest.raises(A.AccerlError):
        A.accerl_actor_forward_mixture(mlp.handle, p3.handle, x, u, np.ones(4, np.uint8), lg, v, a)
    mlp.close(); p3.close()
