"""HIP path vs CPU oracle, element by element, through the C ABI.

Bars: integer accumulators, requantized activations and the int8 student's logits/values (a single
fp32 multiply of an exact accumulator) bit-exact; fp32 teacher 1e-3 and bf16 teacher 2e-2 relative
to the row's largest |logit|; sampled actions identical except where the uniform lies within delta of
a CDF boundary of the oracle's distribution (expf differs by ulps between the two sides).
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import (policies, make_states, rel_err_rows, student_tensors, teacher_tensors, check_actions,
                     check_sampler_self_consistency)

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-3, "bf16": 2e-2}


@pytest.fixture(scope="module")
def A():
    import paper_2211_15023_amd as A
    A.load_library()
    return A


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


_cache = {}


def gpu_policy(A, ci, role):
    key = (ci, role)
    if key not in _cache:
        nt, pt, ns, ps, qp = policies(ci)
        if role == "student":
            _cache[key] = A.Policy(ns, "int8", student_tensors(qp), qp.act_scales)
        else:
            _cache[key] = A.Policy(nt, wl.CONFIGS[ci]["teacher_precision"], teacher_tensors(pt))
    return _cache[key]


def nhwc(x):
    """oracle NCHW tap -> channels-last with channels padded to a multiple of 4"""
    x = np.transpose(x, (0, 2, 3, 1))
    c = x.shape[-1]
    cs = (c + 3) // 4 * 4
    if cs != c:
        x = np.concatenate([x, np.zeros(x.shape[:-1] + (cs - c,), x.dtype)], axis=-1)
    return np.ascontiguousarray(x)


def run_student(A, ci, B, first=0, taps=True):
    nt, pt, ns, ps, qp = policies(ci)
    pol = gpu_policy(A, ci, "student")
    x = make_states(ns, B, wl.STREAM["states"], first)
    u = wl.make_uniforms(B, first)
    print(f"student cfg{ci} B={B} first={first}", flush=True)
    otaps = {}
    ref = oracle.forward_int8(ns, qp, x, u, taps=otaps)
    dx, du = dev(x), dev(u)
    logits, value, action = pol.forward(dx, du)
    torch.cuda.synchronize()
    assert np.array_equal(logits.cpu().numpy(), ref["logits"]), np.abs(logits.cpu().numpy() - ref["logits"]).max()
    assert np.array_equal(value.cpu().numpy(), ref["value"])
    nbad = check_actions(action.cpu().numpy(), ref["action"], ref["logits"], u, 1e-5)
    if taps:
        for (layer, tag), arr in otaps.items():
            if layer == "heads":
                layer_i, kind = len(ns.layers), A.TAP_ACC
            else:
                layer_i = layer
                kind = {"acc": A.TAP_ACC, "act": A.TAP_ACT, "accA": A.TAP_ACC_A, "actA": A.TAP_ACT_A, "accB": A.TAP_ACC}[tag]
            exp = nhwc(arr) if arr.ndim == 4 else arr
            got = pol.tap(dx, layer_i, kind, exp.shape, torch.int32 if exp.dtype == np.int32 else torch.int8)
            g = got.cpu().numpy()
            assert np.array_equal(g, exp), (ci, layer, tag, int((g != exp).sum()), exp.size)
    return nbad


def run_teacher(A, ci, B, first=0):
    nt, pt, ns, ps, qp = policies(ci)
    prec = wl.CONFIGS[ci]["teacher_precision"]
    pol = gpu_policy(A, ci, "teacher")
    x = make_states(nt, B, wl.STREAM["states"], first)
    u = wl.make_uniforms(B, first)
    print(f"teacher cfg{ci} {prec} B={B}", flush=True)
    ref = oracle.forward_float(nt, pt, x, u, prec)
    logits, value, action = pol.forward(dev(x), dev(u))
    torch.cuda.synchronize()
    tol = TOL[prec]
    e = rel_err_rows(logits.cpu().numpy(), ref["logits"]).max()
    assert e <= tol, e
    assert rel_err_rows(value.cpu().numpy(), ref["value"]).max() <= tol
    check_actions(action.cpu().numpy(), ref["action"], ref["logits"], u, 1e-5 if prec == "fp32" else tol)
    # the sampler on its own: the oracle's sampler on the GPU's logits must give the GPU's actions
    check_sampler_self_consistency(action.cpu().numpy(), logits.cpu().numpy(), u)
    return e


@pytest.mark.parametrize("ci,B", [(0, 32), (0, 1), (0, 17), (1, 1024), (1, 1000), (1, 8192)])
def test_mlp_student(A, ci, B):
    run_student(A, ci, B)


@pytest.mark.parametrize("ci,B", [(0, 32), (0, 5), (1, 1024), (1, 77)])
def test_mlp_teacher(A, ci, B):
    run_teacher(A, ci, B)


# config 3 at 1, 21 and 160 states: the residual-block kernel takes 1, 2 or 7 images at a time, so these end in batches
# of one image, of one image short of two, and of six out of seven
@pytest.mark.parametrize("ci,B", [(2, 37), (2, 160), (3, 1), (3, 21), (3, 160)])
def test_cnn_student(A, ci, B):
    run_student(A, ci, B)


@pytest.mark.parametrize("ci,B", [(2, 37), (2, 160), (3, 21), (3, 160)])
def test_cnn_teacher(A, ci, B):
    run_teacher(A, ci, B)


def test_empty_batch_and_errors(A):
    pol = gpu_policy(A, 0, "student")
    z = torch.empty((0, 4), dtype=torch.float32, device="cuda")
    u = torch.empty((0,), dtype=torch.float32, device="cuda")
    out = pol.forward(z, u)
    assert out[0].shape == (0, 2)
    x = dev(make_states(pol.net, 4, wl.STREAM["states"]))
    uu = dev(wl.make_uniforms(4))
    lo, va, ac = pol.alloc_outputs(4)
    with pytest.raises(A.AccerlError):      # student policy through the teacher entry point
        A.accerl_actor_forward_teacher(pol.handle, x, uu, lo, va, ac)
    with pytest.raises(A.AccerlError):      # misaligned output pointer
        big = torch.empty(4 * 2 + 1, dtype=torch.float32, device="cuda")
        A.accerl_actor_forward(pol.handle, x, uu, big[1:].view(4, 2), va, ac)
    with pytest.raises(A.AccerlError):      # recurrent entry point on a feed-forward policy
        A.accerl_actor_forward_recurrent(pol.handle, x, uu, None, None, None, lo, va, ac)


@pytest.mark.parametrize("role", ["student", "teacher"])
def test_recurrent_unroll(A, role):
    """Config 4: a few environment steps with done flags; h and c carried on both sides separately."""
    nt, pt, ns, ps, qp = policies(4)
    net = ns if role == "student" else nt
    pol = gpu_policy(A, 4, role)
    B, T = 37, 4
    h0, c0 = wl.make_hc(B, 256)
    done = wl.make_done(T, B, p=0.2)
    assert done.any()
    h_ref, c_ref = h0.copy(), c0.copy()
    dh, dc = dev(h0), dev(c0)
    for t in range(T):
        print(f"recurrent {role} step {t}", flush=True)
        x = make_states(net, B, wl.STREAM["states"], first=t * B)
        u = wl.make_uniforms(B, first=t * B)
        if role == "student":
            ref = oracle.forward_int8(ns, qp, x, u, h=h_ref, c=c_ref, done=done[t])
        else:
            ref = oracle.forward_float(nt, pt, x, u, "bf16", h=h_ref, c=c_ref, done=done[t])
        h_ref, c_ref = ref["h"], ref["c"]
        logits, value, action = pol.forward(dev(x), dev(u), done=dev(done[t]), h=dh, c=dc)
        torch.cuda.synchronize()
        el = rel_err_rows(logits.cpu().numpy(), ref["logits"])
        ev = rel_err_rows(value.cpu().numpy(), ref["value"]).max()
        eh = np.abs(dh.cpu().numpy() - h_ref).max() / np.abs(h_ref).max()
        ec = np.abs(dc.cpu().numpy() - c_ref).max() / np.abs(c_ref).max()
        print(f"  logits max {el.max():.2e} p90 {np.quantile(el, 0.9):.2e} median {np.median(el):.2e} "
              f"value {ev:.2e} h {eh:.2e} c {ec:.2e}", flush=True)
        # student: the int8 torso is bit-exact, so the bf16 recurrent core sees identical inputs on both
        # sides and only fp32-vs-fp64 accumulation separates them.  teacher: 16 bf16 layers in front of
        # saturating gates amplify single bf16 rounding flips of the torso (an fp32-accumulating CPU
        # implementation deviates from the oracle by 3.5e-2 at most, see test_bf16_noise_floor_cpu), so
        # the 2e-2 bar is applied to the bulk (90th percentile) and 6e-2 to the worst element; h and c within 0.15 of
        # max |ref| (measured 0.107 at most).  test_gpu_recurrent.py::test_bf16_teacher_layer_by_layer holds every
        # kernel of this path, on its own input, to one bf16 rounding and the core to 1e-4.
        if role == "student":
            assert el.max() <= 2e-3 and ev <= 2e-3 and eh <= 1e-4 and ec <= 1e-4
            check_actions(action.cpu().numpy(), ref["action"], ref["logits"], u, 2e-3)
        else:
            assert np.quantile(el, 0.9) <= 2e-2 and el.max() <= 6e-2 and ev <= 6e-2 and eh <= 0.15 and ec <= 0.15
            check_actions(action.cpu().numpy(), ref["action"], ref["logits"], u, 6e-2)
        check_sampler_self_consistency(action.cpu().numpy(), logits.cpu().numpy(), u)
        # carry the oracle's state on the GPU side too, so that each step is compared on equal inputs
        dh.copy_(torch.from_numpy(h_ref))
        dc.copy_(torch.from_numpy(c_ref))
    # rows that were reset at the last step carry no trace of their earlier state
    assert np.isfinite(dh.cpu().numpy()).all()


def test_recurrent_torso_taps_bit_exact(A):
    nt, pt, ns, ps, qp = policies(4)
    pol = gpu_policy(A, 4, "student")
    B = 19
    x = make_states(ns, B, wl.STREAM["states"])
    otaps = {}
    h0, c0 = wl.make_hc(B, 256)
    oracle.forward_int8(ns, qp, x, wl.make_uniforms(B), h=h0, c=c0, taps=otaps)
    i_fc = max(i for i, l in enumerate(ns.layers) if l["kind"] == "dense")
    exp = otaps[(i_fc, "act")]
    got = pol.tap(dev(x), i_fc, A.TAP_ACT, exp.shape, torch.int8).cpu().numpy()
    assert np.array_equal(got, exp)
