"""The paper's own networks (Section 3.1, network table): Original with its printed FC width of 2048,
and the distilled students Net1-Net3, through the same kernels — int8 bit-exact against the oracle
(accumulators, activations, logits), bf16 within the bf16 tolerance.  Net2 and Net3 exercise the
narrow-channel paths (8 and 4 output channels: adjacent output pixels packed into one MFMA tile)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import make_states, rel_err_rows, teacher_tensors, check_actions, check_sampler_self_consistency
from test_gpu_parity import nhwc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2211_15023_amd as A
    A.load_library()
    return A


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


NETS = {
    "original2048": lambda: wl.nature_cnn("original2048", fc=2048),
    "net1": lambda: wl.configs.PAPER_STUDENTS["net1"],
    "net2": lambda: wl.configs.PAPER_STUDENTS["net2"],
    "net3": lambda: wl.configs.PAPER_STUDENTS["net3"],
}


@pytest.mark.parametrize("name,B", [("net1", 37), ("net2", 37), ("net3", 37), ("net3", 160), ("net2", 160), ("original2048", 21)])
def test_paper_net_int8_bit_exact(A, name, B):
    net = NETS[name]()
    params = wl.init_params(net, wl.STREAM["weights_student"])
    qp = oracle.quantize_policy(net, params, make_states(net, 64, wl.STREAM["calibration"]))
    pol = A.Policy(net, "int8", qp.tensors, qp.act_scales)
    x = make_states(net, B, wl.STREAM["states"])
    u = wl.make_uniforms(B)
    print(f"{name} int8 B={B}", flush=True)
    otaps = {}
    ref = oracle.forward_int8(net, qp, x, u, taps=otaps)
    dx = _dev(x)
    logits, value, action = pol.forward(dx, _dev(u))
    torch.cuda.synchronize()
    assert np.array_equal(logits.cpu().numpy(), ref["logits"])
    assert np.array_equal(value.cpu().numpy(), ref["value"])
    check_actions(action.cpu().numpy(), ref["action"], ref["logits"], u, 1e-5)
    for (layer, tag), arr in otaps.items():
        layer_i = len(net.layers) if layer == "heads" else layer
        kind = A.TAP_ACC if (layer == "heads" or tag == "acc") else A.TAP_ACT
        exp = nhwc(arr) if arr.ndim == 4 else arr
        got = pol.tap(dx, layer_i, kind, exp.shape, torch.int32 if exp.dtype == np.int32 else torch.int8).cpu().numpy()
        assert np.array_equal(got, exp), (name, layer, tag, int((got != exp).sum()))
    pol.close()


@pytest.mark.parametrize("name,B", [("net1", 37), ("net2", 37), ("net3", 37), ("original2048", 21)])
def test_paper_net_bf16(A, name, B):
    net = NETS[name]()
    params = wl.init_params(net, wl.STREAM["weights_student"])
    pol = A.Policy(net, "bf16", teacher_tensors(params))
    x = make_states(net, B, wl.STREAM["states"])
    u = wl.make_uniforms(B)
    print(f"{name} bf16 B={B}", flush=True)
    ref = oracle.forward_float(net, params, x, u, "bf16")
    logits, value, action = pol.forward(_dev(x), _dev(u))
    torch.cuda.synchronize()
    assert rel_err_rows(logits.cpu().numpy(), ref["logits"]).max() <= 2e-2
    assert rel_err_rows(value.cpu().numpy(), ref["value"]).max() <= 2e-2
    check_actions(action.cpu().numpy(), ref["action"], ref["logits"], u, 2e-2)
    check_sampler_self_consistency(action.cpu().numpy(), logits.cpu().numpy(), u)
    pol.close()
