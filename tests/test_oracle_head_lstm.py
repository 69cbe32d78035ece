"""Pins for log-softmax, the inverse-CDF sampler and the LSTM cell."""
import numpy as np
import scipy.special
import scipy.stats
import torch

from oracle import layers as L

rng = np.random.default_rng(777)


def test_logsoftmax_rows_sum_to_one_and_library():
    logits = (rng.standard_normal((500, 18)) * 3).astype(np.float32)
    u = rng.random(500).astype(np.float32)
    act, logp = L.softmax_sample(logits, u, want_logp=True)
    p = np.exp(logp.astype(np.float64))
    assert np.abs(p.sum(axis=1) - 1).max() <= 1e-6
    ref = scipy.special.log_softmax(logits.astype(np.float64), axis=1)
    assert np.abs(logp - ref).max() <= 2e-6
    # shift invariance
    _, logp2 = L.softmax_sample(logits + np.float32(8.0), u, want_logp=True)
    assert np.abs(logp2 - logp).max() <= 4e-6
    # two actions: p0 = logistic(l0 - l1)
    l2 = (rng.standard_normal((100, 2)) * 2).astype(np.float32)
    _, lp = L.softmax_sample(l2, rng.random(100).astype(np.float32), want_logp=True)
    assert np.abs(np.exp(lp[:, 0].astype(np.float64)) - scipy.special.expit(l2[:, 0].astype(np.float64) - l2[:, 1])).max() <= 1e-6


def test_sampler_edges():
    logits = np.array([[0.0, 1.0, -1.0, 2.0]], np.float32)
    one = np.nextafter(np.float32(1.0), np.float32(0.0))
    assert L.softmax_sample(logits, np.array([0.0], np.float32))[0] == 0
    assert L.softmax_sample(logits, np.array([one], np.float32))[0] == 3
    # one-hot distribution: that action for every u
    hot = np.full((64, 6), -1e4, np.float32)
    hot[:, 4] = 0.0
    u = np.linspace(0, one, 64).astype(np.float32)
    assert np.all(L.softmax_sample(hot, u) == 4)
    # leading zero-probability action is skipped even at u = 0 (strict cum > u*Z)
    lead = np.array([[-1e4, 0.0, 0.0]], np.float32)
    assert L.softmax_sample(lead, np.array([0.0], np.float32))[0] == 1
    # A = 1
    assert L.softmax_sample(np.zeros((3, 1), np.float32), np.array([0, .5, one], np.float32)).tolist() == [0, 0, 0]


def test_sampler_grid_counts_match_cdf():
    """u on the grid (k+0.5)/N: the count of action a is the number of grid points in
    [cdf_{a-1}, cdf_a), i.e. N*p_a up to +-1."""
    logits = np.array([0.3, -1.2, 2.0, 0.0, -0.5, 1.1], np.float32)
    N = 100000
    u = ((np.arange(N) + 0.5) / N).astype(np.float32)
    act = L.softmax_sample(np.tile(logits, (N, 1)), u)
    p = scipy.special.softmax(logits.astype(np.float64))
    counts = np.bincount(act, minlength=6)
    assert counts.sum() == N
    assert np.abs(counts - N * p).max() <= 2.0, (counts, N * p)
    # the action is non-decreasing in u
    assert np.all(np.diff(act) >= 0)


def test_sampler_frequencies_chi_square():
    logits = (rng.standard_normal(18) * 1.5).astype(np.float32)
    N = 200000
    u = rng.random(N).astype(np.float32)
    act = L.softmax_sample(np.tile(logits, (N, 1)), u)
    p = scipy.special.softmax(logits.astype(np.float64))
    chi2, pval = scipy.stats.chisquare(np.bincount(act, minlength=18), N * p)
    assert pval > 1e-4, (chi2, pval)


def _torch_cell(In, Hd, w_ih, w_hh, b):
    cell = torch.nn.LSTMCell(In, Hd).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(w_ih).double())
        cell.weight_hh.copy_(torch.from_numpy(w_hh).double())
        cell.bias_ih.copy_(torch.from_numpy(b).double())
        cell.bias_hh.zero_()
    return cell


def test_lstm_vs_library_cell():
    B, In, Hd = 5, 12, 7
    x = rng.standard_normal((B, In)).astype(np.float32)
    h = (rng.standard_normal((B, Hd)) * 0.5).astype(np.float32)
    c = (rng.standard_normal((B, Hd)) * 0.5).astype(np.float32)
    w_ih = (rng.standard_normal((4 * Hd, In)) * 0.3).astype(np.float32)
    w_hh = (rng.standard_normal((4 * Hd, Hd)) * 0.3).astype(np.float32)
    b = rng.standard_normal(4 * Hd).astype(np.float32)
    h1, c1 = L.lstm_step(x, h, c, None, w_ih, w_hh, b, False)
    with torch.no_grad():
        hr, cr = _torch_cell(In, Hd, w_ih, w_hh, b)(torch.from_numpy(x).double(),
                                                    (torch.from_numpy(h).double(), torch.from_numpy(c).double()))
    assert np.abs(h1 - hr.numpy()).max() < 2e-6 and np.abs(c1 - cr.numpy()).max() < 2e-6
    # done: rows with done=1 behave as if h = c = 0 had been passed
    done = np.array([1, 0, 1, 0, 0], np.uint8)
    h2, c2 = L.lstm_step(x, h, c, done, w_ih, w_hh, b, False)
    hz, cz = h.copy(), c.copy()
    hz[done == 1] = 0
    cz[done == 1] = 0
    h3, c3 = L.lstm_step(x, hz, cz, None, w_ih, w_hh, b, False)
    assert np.array_equal(h2, h3) and np.array_equal(c2, c3)
    assert np.array_equal(h2[done == 0], h1[done == 0])
    # bf16 operand mode = rounding x, h and both matrices first
    hb, cb = L.lstm_step(x, h, c, None, w_ih, w_hh, b, True)
    hb2, cb2 = L.lstm_step(L.bf16_round(x), L.bf16_round(h), c, None, L.bf16_round(w_ih), L.bf16_round(w_hh), b, False)
    # c is not a GEMM operand and must not be rounded; h enters only through the GEMM
    assert np.array_equal(cb, cb2) and np.array_equal(hb, hb2)


def test_lstm_special_cases():
    B, In, Hd = 3, 4, 5
    x = rng.standard_normal((B, In)).astype(np.float32)
    z = np.zeros((B, Hd), np.float32)
    # zero weights and bias, zero state: gates are sig(0)=.5, tanh(0)=0 -> c = 0, h = 0
    h, c = L.lstm_step(x, z, z, None, np.zeros((4 * Hd, In), np.float32), np.zeros((4 * Hd, Hd), np.float32),
                       np.zeros(4 * Hd, np.float32), False)
    assert not h.any() and not c.any()
    # scalar hand example, In = Hd = 1: gates i,f,g,o from rows 0..3
    w_ih = np.array([[1.0], [2.0], [0.5], [-1.0]], np.float32)
    w_hh = np.array([[0.5], [0.0], [1.0], [2.0]], np.float32)
    b = np.array([0.1, -0.2, 0.3, 0.0], np.float32)
    xs, hs, cs = 0.7, -0.4, 0.9
    sig = lambda v: 1 / (1 + np.exp(-v))
    i_, f_, g_, o_ = (w_ih[k, 0] * xs + w_hh[k, 0] * hs + b[k] for k in range(4))
    c_ref = sig(f_) * cs + sig(i_) * np.tanh(g_)
    h_ref = sig(o_) * np.tanh(c_ref)
    h1, c1 = L.lstm_step(np.array([[xs]], np.float32), np.array([[hs]], np.float32), np.array([[cs]], np.float32),
                         None, w_ih, w_hh, b, False)
    assert abs(h1[0, 0] - h_ref) < 1e-6 and abs(c1[0, 0] - c_ref) < 1e-6
    # done at every step makes an unroll stateless
    T = 4
    xsq = rng.standard_normal((T, B, In)).astype(np.float32)
    w1 = (rng.standard_normal((4 * Hd, In)) * 0.4).astype(np.float32)
    w2 = (rng.standard_normal((4 * Hd, Hd)) * 0.4).astype(np.float32)
    bb = rng.standard_normal(4 * Hd).astype(np.float32)
    h, c = (rng.standard_normal((B, Hd)).astype(np.float32) for _ in range(2))
    ones = np.ones(B, np.uint8)
    for t in range(T):
        h, c = L.lstm_step(xsq[t], h, c, ones, w1, w2, bb, False)
        hf, cf = L.lstm_step(xsq[t], z, z, None, w1, w2, bb, False)
        assert np.array_equal(h, hf) and np.array_equal(c, cf)
