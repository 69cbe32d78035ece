"""Parity on networks that are not among the benchmark configurations: odd image sizes, 3 input channels,
thin layers whose output pixels are packed by 2 and by 4, max-pools fused over several bands, a residual
block on a packed stream, the fused first-two-convolutions kernel with a 16-channel first layer, dense
layers whose K is not a multiple of the MFMA step.  int8: accumulators, activations and logits bit-exact;
bf16: within the bf16 tolerance."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads import Net, conv, dense, maxpool, resblock, relu, flatten
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


def _nets():
    return {
        # 3 planes, non-square; 6 -> 8 stored channels: two output pixels per MFMA tile; pool fused; resblock on the packed stream
        "thin_pool_res": Net("thin_pool_res", "u8", (3, 24, 32), 5, [
            conv(3, 6, 3, 1, 1, False), maxpool(3, 2, 1), resblock(6), relu(), flatten(), dense(6 * 12 * 16, 40, True)]),
        # 4 stored channels: four output pixels per tile (5x5 stride 2), then an unpadded 3x3 to 12 channels, odd sizes
        "pack4": Net("pack4", "u8", (4, 36, 36), 7, [
            conv(4, 4, 5, 2, 2, True), conv(4, 12, 3, 1, 0, True), flatten(), dense(12 * 16 * 16, 50, True)]),
        # tall image: the pooled first layer runs in several bands; 16 and 20 channels (no packing), pool after a ReLU conv
        "bands": Net("bands", "u8", (2, 120, 16), 4, [
            conv(2, 16, 3, 1, 1, True), maxpool(3, 2, 1), conv(16, 20, 3, 1, 1, False), maxpool(3, 2, 1),
            relu(), flatten(), dense(20 * 30 * 4, 33, True)]),
        # 40 actions: three head tiles, the heads kernel stages its logits in LDS and scans them with one lane per state
        "many_actions": Net("many_actions", "u8", (4, 20, 20), 40, [
            conv(4, 16, 4, 2, 0, True), flatten(), dense(16 * 9 * 9, 64, True)]),
        # the fused first-two-convolutions kernel with one channel tile in the first layer
        "fused16": Net("fused16", "u8", (4, 60, 60), 6, [
            conv(4, 16, 8, 4, 0, True), conv(16, 64, 4, 2, 0, True), flatten(), dense(64 * 6 * 6, 24, False)]),
    }


@pytest.mark.parametrize("name", ["thin_pool_res", "pack4", "bands", "fused16", "many_actions"])
@pytest.mark.parametrize("B", [5, 67])
def test_int8_bit_exact_with_taps(A, name, B):
    net = _nets()[name]
    params = wl.init_params(net, wl.STREAM["weights_student"])
    qp = oracle.quantize_policy(net, params, make_states(net, 32, wl.STREAM["calibration"]))
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
        kind = {"acc": A.TAP_ACC, "act": A.TAP_ACT, "accA": A.TAP_ACC_A, "actA": A.TAP_ACT_A, "accB": A.TAP_ACC}[tag]
        if layer == "heads":
            kind = A.TAP_ACC
        exp = nhwc(arr) if arr.ndim == 4 else arr
        got = pol.tap(dx, layer_i, kind, exp.shape, torch.int32 if exp.dtype == np.int32 else torch.int8).cpu().numpy()
        assert np.array_equal(got, exp), (name, layer, tag, int((got != exp).sum()))
    pol.close()


@pytest.mark.parametrize("name", ["thin_pool_res", "pack4", "bands", "fused16", "many_actions"])
def test_bf16_within_tolerance(A, name):
    net = _nets()[name]
    B = 19
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


def _mlps():
    d = wl.dense
    return {
        # 40 features: the first layer on the K = 64 MFMA (16 features per lane); 6 actions: sampler in registers
        "wide_obs": Net("wide_obs", "f32", (40,), 6, [d(40, 48, True), d(48, 64, True)]),
        # 20 actions: two head tiles, logits staged in LDS and scanned by one lane per state
        "many_actions": Net("many_actions", "f32", (24,), 20, [d(24, 64, True)]),
        # 7 features (rows are not whole 16-byte groups: scalar observation loads), a hidden layer without ReLU
        # (signed requantization, first-layer layout chosen at run time), 3 actions
        "odd_obs_no_relu": Net("odd_obs_no_relu", "f32", (7,), 3, [d(7, 32, True), d(32, 16, False)]),
        # three hidden layers, 64 features, the most actions the register sampler takes
        "deep_15": Net("deep_15", "f32", (64,), 15, [d(64, 64, True), d(64, 64, True), d(64, 64, True)]),
    }


@pytest.mark.parametrize("name", ["wide_obs", "many_actions", "odd_obs_no_relu", "deep_15"])
@pytest.mark.parametrize("B", [1, 333])
def test_mlp_variants_bit_exact_with_taps(A, name, B):
    """The fused MLP kernel's variants beyond the two benchmark networks, accumulators and activations bit-exact."""
    net = _mlps()[name]
    params = wl.init_params(net, wl.STREAM["weights_student"])
    qp = oracle.quantize_policy(net, params, make_states(net, 256, wl.STREAM["calibration"]))
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
        kind = A.TAP_ACC if tag == "acc" or layer == "heads" else A.TAP_ACT
        got = pol.tap(dx, layer_i, kind, arr.shape, torch.int32 if arr.dtype == np.int32 else torch.int8).cpu().numpy()
        assert np.array_equal(got, arr), (name, layer, tag, int((got != arr).sum()))
    pol.close()
