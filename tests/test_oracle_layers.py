"""Pins for the oracle's layer functions: brute force, library routines, closed forms."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import layers as L

rng = np.random.default_rng(12345)


def brute_conv(x, w, b, s, p):
    """Seven nested Python loops over Python ints / floats."""
    B, C, H, W = x.shape
    Co, _, k, _ = w.shape
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    y = [[[[None] * Wo for _ in range(Ho)] for _ in range(Co)] for _ in range(B)]
    for n in range(B):
        for co in range(Co):
            for oy in range(Ho):
                for ox in range(Wo):
                    acc = b[co].item()
                    for ci in range(C):
                        for ky in range(k):
                            for kx in range(k):
                                iy, ix = oy * s + ky - p, ox * s + kx - p
                                if 0 <= iy < H and 0 <= ix < W:
                                    acc += w[co, ci, ky, kx].item() * x[n, ci, iy, ix].item()
                    y[n][co][oy][ox] = acc
    return np.array(y)


CONV_CASES = [(1, 2, 5, 5, 3, 3, 1, 0), (1, 2, 5, 5, 3, 3, 1, 1), (2, 3, 7, 6, 4, 3, 2, 1),
              (1, 1, 8, 8, 2, 4, 2, 0), (2, 4, 9, 9, 5, 8, 4, 0), (1, 3, 4, 4, 2, 3, 2, 1)]


@pytest.mark.parametrize("B,C,H,W,Co,k,s,p", CONV_CASES)
def test_conv_int_acc_vs_brute_force(B, C, H, W, Co, k, s, p):
    for is_u8 in (False, True):
        x = rng.integers(0, 256, (B, C, H, W)).astype(np.uint8) if is_u8 else \
            rng.integers(-127, 128, (B, C, H, W)).astype(np.int8)
        w = rng.integers(-127, 128, (Co, C, k, k)).astype(np.int8)
        b = rng.integers(-5000, 5000, Co).astype(np.int32)
        got = L.conv2d_q_acc(x, w, b, s, p)
        ref = brute_conv(x.astype(np.int64), w.astype(np.int64), b.astype(np.int64), s, p)
        assert got.dtype == np.int32 and np.array_equal(got, ref)


@pytest.mark.parametrize("B,C,H,W,Co,k,s,p", CONV_CASES)
def test_conv_int_acc_vs_library_conv(B, C, H, W, Co, k, s, p):
    x = rng.integers(-127, 128, (B, C, H, W)).astype(np.int8)
    w = rng.integers(-127, 128, (Co, C, k, k)).astype(np.int8)
    b = rng.integers(-5000, 5000, Co).astype(np.int32)
    ref = F.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                   torch.from_numpy(b.astype(np.float64)), stride=s, padding=p).numpy()
    assert np.array_equal(L.conv2d_q_acc(x, w, b, s, p), ref.astype(np.int64))
    # relu on load = conv of max(x, 0)
    ref_r = F.conv2d(torch.from_numpy(np.maximum(x, 0).astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                     torch.from_numpy(b.astype(np.float64)), stride=s, padding=p).numpy()
    assert np.array_equal(L.conv2d_q_acc(x, w, b, s, p, relu_in=True), ref_r.astype(np.int64))


@pytest.mark.parametrize("B,C,H,W,Co,k,s,p", CONV_CASES)
@pytest.mark.parametrize("relu", [False, True])
def test_conv_float_vs_library_and_brute(B, C, H, W, Co, k, s, p, relu):
    x = rng.standard_normal((B, C, H, W)).astype(np.float32)
    w = rng.standard_normal((Co, C, k, k)).astype(np.float32)
    b = rng.standard_normal(Co).astype(np.float32)
    ref = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), torch.from_numpy(b).double(),
                   stride=s, padding=p)
    if relu:
        ref = ref.clamp_min(0)
    got = L.conv2d_f(x, w, b, s, p, relu, False)
    np.testing.assert_allclose(got, ref.numpy(), rtol=0, atol=4e-6 * np.abs(ref.numpy()).max())
    bf = brute_conv(x.astype(np.float64), w.astype(np.float64), b.astype(np.float64), s, p)
    if relu:
        bf = np.maximum(bf, 0)
    np.testing.assert_allclose(got, bf, rtol=0, atol=4e-6 * np.abs(bf).max())


def test_conv_asymmetric_input_catches_transposition():
    # a single 1 in the kernel picks one shifted copy of the image: fixes ky/kx and iy/ix roles
    x = np.arange(1 * 1 * 4 * 5, dtype=np.int8).reshape(1, 1, 4, 5)
    w = np.zeros((1, 1, 2, 3), np.int8)
    # k must be square in the oracle: embed in 3x3
    w = np.zeros((1, 1, 3, 3), np.int8)
    w[0, 0, 0, 2] = 1                                      # ky=0, kx=2
    acc = L.conv2d_q_acc(x, w, np.zeros(1, np.int32), 1, 0)
    assert np.array_equal(acc[0, 0], x[0, 0, 0:2, 2:5].astype(np.int32))
    w[:] = 0
    w[0, 0, 2, 0] = 1                                      # ky=2, kx=0
    acc = L.conv2d_q_acc(x, w, np.zeros(1, np.int32), 1, 0)
    assert np.array_equal(acc[0, 0], x[0, 0, 2:4, 0:3].astype(np.int32))


def test_dense_vs_matmul_and_1x1_conv():
    x = rng.integers(-127, 128, (7, 33)).astype(np.int8)
    w = rng.integers(-127, 128, (5, 33)).astype(np.int8)
    b = rng.integers(-1000, 1000, 5).astype(np.int32)
    ref = x.astype(np.int64) @ w.astype(np.int64).T + b
    assert np.array_equal(L.dense_q_acc(x, w, b), ref)
    assert np.array_equal(L.dense_q_acc(x, w, b, relu_in=True), np.maximum(x, 0).astype(np.int64) @ w.astype(np.int64).T + b)
    # a 1x1 convolution over a 1x1 image is the dense layer
    acc = L.conv2d_q_acc(x.reshape(7, 33, 1, 1), w.reshape(5, 33, 1, 1), b, 1, 0)
    assert np.array_equal(acc.reshape(7, 5), ref)
    xf = rng.standard_normal((7, 33)).astype(np.float32)
    wf = rng.standard_normal((5, 33)).astype(np.float32)
    bf = rng.standard_normal(5).astype(np.float32)
    reff = xf.astype(np.float64) @ wf.astype(np.float64).T + bf
    np.testing.assert_allclose(L.dense_f(xf, wf, bf, False, False), reff, rtol=0, atol=2e-6 * np.abs(reff).max())
    np.testing.assert_allclose(L.dense_f(xf, wf, bf, True, False), np.maximum(reff, 0), rtol=0, atol=2e-6 * np.abs(reff).max())
    got = L.conv2d_f(xf.reshape(7, 33, 1, 1), wf.reshape(5, 33, 1, 1), bf, 1, 0, False, False)
    assert np.array_equal(got.reshape(7, 5), L.dense_f(xf, wf, bf, False, False))


def test_quantize_roundtrip_ties_saturation_monotone():
    s = np.float32(0.05)
    inv = np.float32(1.0 / np.float64(s))
    x = np.linspace(-127 * s, 127 * s, 20001).astype(np.float32)
    q = L.quantize_f32(x, inv)
    # error bound s/2 (plus the rounding of x*inv_s in fp32)
    assert np.abs(x.astype(np.float64) - q.astype(np.float64) * np.float64(s)).max() <= s / 2 * (1 + 1e-5)
    assert np.all(np.diff(q.astype(np.int32)) >= 0)
    # saturation
    assert L.quantize_f32(np.array([1e9, -1e9, 127.4 * s, 128 * s, -200 * s], np.float32), inv).tolist() == [127, -127, 127, 127, -127]
    # exact ties round to even
    ties = np.array([0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 126.5], np.float32)
    assert L.quantize_f32(ties, np.float32(1.0)).tolist() == [0, 2, 2, 4, 0, -2, -2, 126]


def test_requant_hand_examples():
    # acc * m = 2.5, 3.5, -2.5 -> ties to even 2, 4, -2 ; ReLU clamp lo=0 ; saturation
    acc = np.array([[[5], [7], [-5], [100000], [-100000], [3]]], np.int32).reshape(1, 6, 1)
    m = np.array([0.5, 0.5, 0.5, 0.5, 0.5, 0.25], np.float32)
    assert L.requant(acc, m, -127).reshape(-1).tolist() == [2, 4, -2, 127, -127, 1]
    assert L.requant(acc, m, 0).reshape(-1).tolist() == [2, 4, 0, 127, 0, 1]
    # channel index, not position, selects the multiplier: [B=1, C=2, HW=3]
    acc = np.array([[[10, 20, 30], [10, 20, 30]]], np.int32)
    m = np.array([0.1, 1.0], np.float32)
    assert L.requant(acc, m, -127).tolist() == [[[1, 2, 3], [10, 20, 30]]]
    # monotone in acc for positive m
    a = np.arange(-3000, 3000, dtype=np.int32).reshape(1, 1, -1)
    q = L.requant(a, np.array([0.043], np.float32), -127)
    assert np.all(np.diff(q.reshape(-1).astype(int)) >= 0)


def test_requant_residual_hand_examples():
    # y = fma(acc, m, x*r): acc=4, m=0.25, x=3, r=0.5 -> 1 + 1.5 = 2.5 -> 2 ; x=-3 -> 1-1.5=-0.5 -> -0
    acc = np.array([4, 4, 1000, -1000], np.int32).reshape(1, 1, 4)
    xq = np.array([3, -3, 100, -100], np.int8).reshape(1, 1, 4)
    q = L.requant_residual(acc, xq, np.float32(0.5), np.array([0.25], np.float32))
    assert q.reshape(-1).tolist() == [2, 0, 127, -127]
    # zero branch: output is the stream rescaled by r; identity when r == 1
    xq = rng.integers(-127, 128, (2, 3, 5)).astype(np.int8)
    z = np.zeros((2, 3, 5), np.int32)
    m = np.array([0.3, 0.2, 0.1], np.float32)
    assert np.array_equal(L.requant_residual(z, xq, np.float32(1.0), m), xq)
    exp = np.clip(np.rint(xq.astype(np.float32) * np.float32(0.37)), -127, 127).astype(np.int8)
    assert np.array_equal(L.requant_residual(z, xq, np.float32(0.37), m), exp)


def test_requant_residual_is_single_rounding_fma():
    """y must equal the exactly computed acc*m + t rounded once to fp32 (t = fp32(x*r))."""
    from fractions import Fraction
    n = 4000
    acc = rng.integers(-3000, 3000, n).astype(np.int32)
    xq = rng.integers(-127, 128, n).astype(np.int8)
    m = np.float32(0.0123456789)
    r = np.float32(0.7654321)
    got = L.requant_residual(acc.reshape(1, 1, n), xq.reshape(1, 1, n), r, np.array([m], np.float32)).reshape(-1)
    n_diff = 0
    for i in range(n):
        t = np.float32(np.float32(xq[i]) * r)
        exact = Fraction(int(acc[i])) * Fraction(float(m)) + Fraction(float(t))
        y = np.float32(float(exact))                 # double is exact enough: one further rounding to fp32
        q = int(np.clip(np.rint(y), -127, 127))
        assert got[i] == q, (i, acc[i], xq[i], got[i], q)
        y2 = np.float32(np.float32(acc[i]) * m) + t  # two roundings
        n_diff += int(y2 != y)
    assert n_diff > 0                                # the sample does contain cases where fusing matters


def test_maxpool_brute_library_and_ignore_padding():
    x = rng.integers(-127, 128, (2, 3, 9, 8)).astype(np.int8)
    got = L.maxpool_i8(x, 3, 2, 1)
    ref = F.max_pool2d(torch.from_numpy(x.astype(np.float32)), 3, 2, 1).numpy()   # pads with -inf
    assert got.shape == (2, 3, 5, 4) and np.array_equal(got, ref.astype(np.int8))
    # all-negative map: zero padding would give 0 at the border, ignoring the padding must not
    neg = -np.abs(x) - 1
    neg = np.clip(neg, -127, -1).astype(np.int8)
    g = L.maxpool_i8(neg, 3, 2, 1)
    assert g.max() < 0
    for (oy, ox) in itertools.product(range(5), range(4)):
        win = neg[:, :, max(0, 2 * oy - 1):min(9, 2 * oy + 2), max(0, 2 * ox - 1):min(8, 2 * ox + 2)]
        assert np.array_equal(g[:, :, oy, ox], win.max(axis=(2, 3)))
    xf = rng.standard_normal((2, 3, 9, 8)).astype(np.float32)
    assert np.array_equal(L.maxpool_f(xf, 3, 2, 1), F.max_pool2d(torch.from_numpy(xf), 3, 2, 1).numpy())
    # sizes of the IMPALA torso: 84 -> 42 -> 21 -> 11
    h = 84
    for exp in (42, 21, 11):
        h = L.maxpool_i8(np.zeros((1, 1, h, h), np.int8), 3, 2, 1).shape[-1]
        assert h == exp


def test_maxpool_commutes_with_requant():
    acc = rng.integers(-40000, 40000, (2, 4, 11, 11)).astype(np.int32)
    m = rng.uniform(1e-3, 5e-3, 4).astype(np.float32)
    a = L.maxpool_i8(L.requant(acc, m, -127), 3, 2, 1)
    pooled = F.max_pool2d(torch.from_numpy(acc.astype(np.float64)), 3, 2, 1).numpy().astype(np.int32)
    b = L.requant(pooled, m, -127)
    assert np.array_equal(a, b)


def test_dequant():
    acc = np.array([[3, -7], [100, 0]], np.int32)
    d = np.array([0.5, 0.25], np.float32)
    assert L.dequant(acc, d).tolist() == [[1.5, -1.75], [50.0, 0.0]]
    assert L.dequant_i8(np.array([-4, 8], np.int8), np.float32(0.125)).tolist() == [-0.5, 1.0]


def test_bf16_round_all_patterns_and_library():
    # every bf16 value is a fixed point
    hi = np.arange(65536, dtype=np.uint32) << 16
    f = hi.view(np.float32)
    finite = np.isfinite(f)
    r = L.bf16_round(f)
    assert np.array_equal(r.view(np.uint32)[finite], hi[finite])
    # ties to even: 1 + 2^-8 is halfway between 1 and 1+2^-7 -> 1 ; 1 + 3*2^-8 -> 1 + 2^-6
    assert L.bf16_round(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20], np.float32)).tolist() == \
        [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7]
    # library conversion on random floats, incl. large and tiny magnitudes
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-30, 30, 200000))).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(L.bf16_round(x), ref)


def test_bf16_operand_mode_is_rounding_of_operands():
    x = rng.standard_normal((3, 2, 6, 6)).astype(np.float32)
    w = rng.standard_normal((4, 2, 3, 3)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    a = L.conv2d_f(x, w, b, 1, 1, True, True)
    ref = L.conv2d_f(L.bf16_round(x), L.bf16_round(w), b, 1, 1, True, False)
    assert np.array_equal(a, ref)
    xd = rng.standard_normal((3, 40)).astype(np.float32)
    wd = rng.standard_normal((4, 40)).astype(np.float32)
    assert np.array_equal(L.dense_f(xd, wd, b, False, True), L.dense_f(L.bf16_round(xd), L.bf16_round(wd), b, False, False))
    assert not np.array_equal(L.dense_f(xd, wd, b, False, True), L.dense_f(xd, wd, b, False, False))
