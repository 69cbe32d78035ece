"""Pins of the oracle's Monitor indicators (Monitor section, KL equation) and V-trace
corrector (Corrector section, V-trace equation) against closed forms, library routines,
special cases and an independent restatement."""
import numpy as np
import scipy.special as sps
import scipy.stats as sst

import workloads as wl
from oracle import layers as L


def _softmax64(l):
    l = np.asarray(l, np.float64)
    e = np.exp(l - l.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


# ------------------------------------------------------------------ KL monitor
def test_kl_identical_policies_is_zero_and_shift_invariant():
    lo, _ = wl.make_logits_pair(64, 18)
    kl, ent, st = L.kl_monitor(lo, lo)
    assert np.all(np.abs(kl) < 1e-15)
    assert st[0] == 0.0 or abs(st[0]) < 1e-15
    # adding a constant per row to either table changes nothing (softmax is shift invariant)
    _, ls = wl.make_logits_pair(64, 18)
    shift = np.linspace(-3, 3, 64, dtype=np.float32)[:, None]
    a = L.kl_monitor(lo, ls)
    b = L.kl_monitor(lo + shift, ls - shift)
    assert np.allclose(a[0], b[0], rtol=0, atol=2e-6)      # fp32 rounding of the shifted logits
    assert np.allclose(a[1], b[1], rtol=0, atol=2e-6)


def test_kl_two_actions_closed_form():
    # A = 2: pi(0) = sigmoid(l0 - l1); KL = p log(p/q) + (1-p) log((1-p)/(1-q))
    lo = np.array([[0.3, -1.2], [2.0, 2.0], [-4.0, 1.0]], np.float32)
    ls = np.array([[1.0, 0.5], [0.0, 3.0], [-4.0, 1.0]], np.float32)
    p = sps.expit(lo[:, 0].astype(np.float64) - lo[:, 1])
    q = sps.expit(ls[:, 0].astype(np.float64) - ls[:, 1])
    want = p * np.log(p / q) + (1 - p) * np.log((1 - p) / (1 - q))
    hq = -(q * np.log(q) + (1 - q) * np.log(1 - q))
    kl, ent, st = L.kl_monitor(lo, ls)
    assert np.allclose(kl, want, rtol=1e-12, atol=1e-15)
    assert np.allclose(ent, hq, rtol=1e-12)


def test_kl_matches_library_and_direction():
    lo, ls = wl.make_logits_pair(200, 18, gap=0.8)
    po, ps = _softmax64(lo), _softmax64(ls)
    want = sps.rel_entr(po, ps).sum(axis=1)          # KL(original || smaller), the paper's direction
    rev = sps.rel_entr(ps, po).sum(axis=1)
    kl, ent, st = L.kl_monitor(lo, ls)
    assert np.allclose(kl, want, rtol=1e-10, atol=1e-14)
    assert not np.allclose(kl, rev, rtol=1e-3)       # a swapped direction would fail here
    assert np.all(kl >= -1e-15)
    assert np.allclose(ent, sst.entropy(ps, axis=1), rtol=1e-10)
    assert np.isclose(st[0], want.mean(), rtol=1e-12)
    assert np.isclose(st[1], want.max(), rtol=1e-12)
    assert np.isclose(st[2], want.var(), rtol=1e-9)  # population variance
    assert np.isclose(st[3], sst.entropy(ps, axis=1).mean(), rtol=1e-12)


def test_kl_uniform_against_peaked():
    A = 6
    lo = np.zeros((1, A), np.float32)                       # uniform original
    ls = np.array([[10.0, 0, 0, 0, 0, 0]], np.float32)     # peaked smaller
    kl, ent, _ = L.kl_monitor(lo, ls)
    lq = np.log(_softmax64(ls))[0]
    assert np.isclose(kl[0], -np.log(A) - lq.mean(), rtol=1e-12)
    kl2, ent2, _ = L.kl_monitor(ls, lo)
    assert np.isclose(ent2[0], np.log(A), rtol=1e-12)       # entropy of the uniform policy


# ------------------------------------------------------------------ V-trace
def _traj(T=7, B=5, A=4, **kw):
    return wl.make_trajectory(T, B, A, **kw)


def test_vtrace_on_policy_is_the_bootstrapped_return():
    # pi_original == pi_smaller and rho_bar = c_bar = 1: rho = c = 1, so
    # v_s = sum_{t>=s} (prod_{i<t} gamma_i) r_t + (prod all gamma) V(x_T)
    tr = _traj()
    tr["logits_smaller"] = tr["logits_original"].copy()
    vs, adv, rho = L.vtrace(**tr)
    T, B = tr["rewards"].shape
    want = np.empty((T, B))
    nxt = tr["bootstrap"].astype(np.float64)
    for t in range(T - 1, -1, -1):
        nxt = tr["rewards"][t].astype(np.float64) + tr["discounts"][t].astype(np.float64) * nxt
        want[t] = nxt
    assert np.allclose(rho, 1.0, atol=1e-15)
    assert np.allclose(vs, want, rtol=1e-12, atol=1e-12)


def test_vtrace_zero_clipping_returns_the_values():
    tr = _traj()
    vs, adv, rho = L.vtrace(**tr, rho_bar=0.0, c_bar=0.0)
    assert np.array_equal(vs, tr["values"].astype(np.float64))
    assert np.all(adv == 0.0) and np.all(rho == 0.0)


def test_vtrace_single_step_by_hand():
    lo = np.log(np.array([[[0.5, 0.5]]], np.float32))
    ls = np.log(np.array([[[0.8, 0.2]]], np.float32))
    kw = dict(actions=np.array([[0]], np.int32), rewards=np.array([[2.0]], np.float32),
              discounts=np.array([[0.9]], np.float32), values=np.array([[1.0]], np.float32),
              bootstrap=np.array([3.0], np.float32))
    # ratio = 0.5 / 0.8 = 0.625 < 1;  delta = 0.625 * (2 + 0.9*3 - 1) = 2.3125
    vs, adv, rho = L.vtrace(lo, ls, **kw)
    assert np.isclose(rho[0, 0], 0.625, rtol=1e-6)
    assert np.isclose(vs[0, 0], 1.0 + 0.625 * (2.0 + np.float64(np.float32(0.9)) * 3.0 - 1.0), rtol=1e-6)
    assert np.isclose(adv[0, 0], vs[0, 0] - 1.0, rtol=1e-9)   # T = 1: v_{t+1} is the bootstrap value
    # action 1: ratio = 0.5 / 0.2 = 2.5, clipped at rho_bar = 1
    kw["actions"] = np.array([[1]], np.int32)
    vs, adv, rho = L.vtrace(lo, ls, **kw)
    assert rho[0, 0] == 1.0
    vs2, _, rho2 = L.vtrace(lo, ls, **kw, rho_bar=4.0, c_bar=4.0)
    assert np.isclose(rho2[0, 0], 2.5, rtol=1e-6)


def test_vtrace_sum_form_equals_backward_recurrence():
    # independent restatement: v_s - V(x_s) = delta_s + gamma_s c_s (v_{s+1} - V(x_{s+1}))
    tr = _traj(T=16, B=9, A=6)
    for rb, cb in ((1.0, 1.0), (1.5, 0.7)):
        vs, adv, rho = L.vtrace(**tr, rho_bar=rb, c_bar=cb)
        T, B = tr["rewards"].shape
        lpo = np.log(_softmax64(tr["logits_original"]))
        lps = np.log(_softmax64(tr["logits_smaller"]))
        idx = tr["actions"][..., None].astype(np.int64)
        ratio = np.exp(np.take_along_axis(lpo, idx, 2) - np.take_along_axis(lps, idx, 2))[..., 0]
        r_, c_ = np.minimum(rb, ratio), np.minimum(cb, ratio)
        V = tr["values"].astype(np.float64)
        g = tr["discounts"].astype(np.float64)
        vnext = np.vstack([V[1:], tr["bootstrap"][None].astype(np.float64)])
        delta = r_ * (tr["rewards"] + g * vnext - V)
        acc = np.zeros(B)
        want = np.empty((T, B))
        for t in range(T - 1, -1, -1):
            acc = delta[t] + g[t] * c_[t] * acc
            want[t] = V[t] + acc
        assert np.allclose(rho, r_, rtol=1e-12)
        assert np.allclose(vs, want, rtol=1e-11, atol=1e-12)
        vs_next = np.vstack([want[1:], tr["bootstrap"][None].astype(np.float64)])
        assert np.allclose(adv, r_ * (tr["rewards"] + g * vs_next - V), rtol=1e-10, atol=1e-12)


def test_vtrace_episode_end_cuts_the_trace():
    # a zero discount at step k: nothing after k reaches v_s for s <= k
    tr = _traj(T=8, B=3, A=4, p_done=0.0)
    tr["discounts"][4, :] = 0.0
    vs, _, _ = L.vtrace(**tr)
    tr2 = {k: v.copy() for k, v in tr.items()}
    tr2["rewards"][5:] += 7.0
    tr2["values"][5:] -= 3.0
    tr2["bootstrap"] += 11.0
    vs2, _, _ = L.vtrace(**tr2)
    assert np.array_equal(vs[:5], vs2[:5])
    assert not np.allclose(vs[5:], vs2[5:])


# ------------------------------------------------------------------ distillation loss (Section 2.2 Eq. 1)
def test_distill_loss_terms():
    B, A = 50, 6
    lo, ls = wl.make_logits_pair(B, A, gap=0.6)
    vo = wl.normal(wl.BASE_SEED, 77, 0, B)
    vs = wl.normal(wl.BASE_SEED, 78, 0, B)
    po, ps = _softmax64(lo), _softmax64(ls)
    kl = sps.rel_entr(po, ps).sum(axis=1)
    H = sst.entropy(ps, axis=1)
    for beta in (0.0, 0.01, 1.0):
        loss, mean = L.distill_loss(lo, ls, vo, vs, beta)
        want = kl + 0.5 * (vo.astype(np.float64) - vs) ** 2 - beta * H
        assert np.allclose(loss, want, rtol=1e-10, atol=1e-13)
        assert np.isclose(mean, want.mean(), rtol=1e-12)
    # identical networks: only the entropy bonus is left; the sign of each term is pinned by a one-term change
    loss, _ = L.distill_loss(lo, lo, vo, vo, 0.5)
    assert np.allclose(loss, -0.5 * sst.entropy(po, axis=1), rtol=1e-10)
    l0, _ = L.distill_loss(lo, ls, vo, vo, 0.0)
    l1, _ = L.distill_loss(lo, ls, vo, vo + np.float32(2.0), 0.0)
    assert np.allclose(l1 - l0, 2.0, rtol=1e-6)              # (2)^2 / 2
    # two actions, by hand: p = (.5,.5), q = (.8,.2), dv = 1, beta = .1
    lo2 = np.log(np.array([[0.5, 0.5]], np.float32)); ls2 = np.log(np.array([[0.8, 0.2]], np.float32))
    loss, _ = L.distill_loss(lo2, ls2, np.array([1.0], np.float32), np.array([0.0], np.float32), 0.1)
    klh = 0.5 * np.log(0.5 / 0.8) + 0.5 * np.log(0.5 / 0.2)
    hh = -(0.8 * np.log(0.8) + 0.2 * np.log(0.2))
    assert np.isclose(loss[0], klh + 0.5 - 0.1 * hh, rtol=1e-6)


# ------------------------------------------------------------------ alpha mixture (Section 3.2)
def test_mixture_alpha_schedule():
    assert L.mixture_alpha(0.0, 0.1, 0.5) == 1.0 and L.mixture_alpha(0.1, 0.1, 0.5) == 1.0
    assert L.mixture_alpha(0.5, 0.1, 0.5) == 0.0 and L.mixture_alpha(9.0, 0.1, 0.5) == 0.0
    assert np.isclose(L.mixture_alpha(0.3, 0.1, 0.5), 0.5)
    ks = np.linspace(0.1, 0.5, 9)
    al = np.array([L.mixture_alpha(k, 0.1, 0.5) for k in ks])
    assert np.all(np.diff(al) < 0) and np.allclose(np.diff(al), np.diff(al)[0])    # decreasing, linear
