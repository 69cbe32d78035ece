"""GPU parity of the Monitor indicators and the V-trace corrector against the fp64 oracle.

Tolerances: the kernels work in fp32 per row (expf/logf, sums of at most 64 terms), the oracle in
fp64 — far inside the 1e-3 relative bound stated for fp32 paths; the bounds below are what the
arithmetic gives (a few fp32 ulps per term, times A terms, times T steps for the scan)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import layers as L

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    import paper_2211_15023_amd as A
    A.load_library()
    return A


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


@pytest.mark.parametrize("B,nA", [(1, 2), (63, 18), (64, 18), (4096 + 17, 18), (1000, 64), (777, 7), (300, 32)])
def test_kl_monitor_matches_oracle(A, B, nA):
    lo, ls = wl.make_logits_pair(B, nA, gap=0.5)
    kl_o, ent_o, st_o = L.kl_monitor(lo, ls)
    kl = torch.empty(B, dtype=torch.float32, device="cuda")
    ent = torch.empty(B, dtype=torch.float32, device="cuda")
    st = torch.zeros(4, dtype=torch.float64, device="cuda")
    A.accerl_monitor_kl(_dev(lo), _dev(ls), kl, ent, st)
    torch.cuda.synchronize()
    assert np.allclose(kl.cpu().numpy(), kl_o, rtol=2e-4, atol=3e-6)
    assert np.allclose(ent.cpu().numpy(), ent_o, rtol=2e-5, atol=3e-6)
    got = st.cpu().numpy()
    assert np.isclose(got[0], st_o[0], rtol=1e-4, atol=1e-6)
    assert np.isclose(got[1], st_o[1], rtol=2e-4, atol=3e-6)
    assert np.isclose(got[2], st_o[2], rtol=1e-3, atol=1e-7)
    assert np.isclose(got[3], st_o[3], rtol=1e-5)
    # outputs are optional
    st2 = torch.zeros(4, dtype=torch.float64, device="cuda")
    A.accerl_monitor_kl(_dev(lo), _dev(ls), None, None, st2)
    torch.cuda.synchronize()
    assert np.array_equal(st2.cpu().numpy(), got)          # fixed reduction order: same bits


def test_kl_monitor_identical_policies(A):
    lo, _ = wl.make_logits_pair(500, 18)
    st = torch.ones(4, dtype=torch.float64, device="cuda")
    kl = torch.empty(500, dtype=torch.float32, device="cuda")
    A.accerl_monitor_kl(_dev(lo), _dev(lo), kl, None, st)
    torch.cuda.synchronize()
    assert float(kl.abs().max()) == 0.0
    assert st.cpu().numpy()[:3].tolist() == [0.0, 0.0, 0.0]


def test_kl_monitor_large_batch_stats(A):
    # the size of one monitoring pass over a full unroll: 16 steps x 4096 environments
    B, nA = 16 * 4096, 18
    lo, ls = wl.make_logits_pair(B, nA)
    _, _, st_o = L.kl_monitor(lo, ls)
    st = torch.zeros(4, dtype=torch.float64, device="cuda")
    A.accerl_monitor_kl(_dev(lo), _dev(ls), None, None, st)
    torch.cuda.synchronize()
    assert np.allclose(st.cpu().numpy(), st_o, rtol=2e-4, atol=1e-6)


# the scan splits a trajectory into runs of 4 steps (T <= 32) or 16 steps handled by different wavefronts, and walks
# unrolls of more than 256 steps in several rounds: 40 and 257 steps end in a cut run, 300 and 257 need a second round
@pytest.mark.parametrize("T,B,nA,rb,cb", [(1, 1, 2, 1.0, 1.0), (16, 300, 18, 1.0, 1.0), (20, 257, 6, 1.5, 0.8),
                                         (5, 4096, 18, 1.0, 1.0), (64, 33, 64, 2.0, 1.0), (40, 65, 4, 1.0, 0.9),
                                         (257, 64, 3, 1.0, 1.0), (300, 70, 5, 1.2, 1.0), (32, 64, 18, 1.0, 1.0), (33, 5, 18, 1.0, 1.0)])
def test_vtrace_matches_oracle(A, T, B, nA, rb, cb):
    tr = wl.make_trajectory(T, B, nA, p_done=0.05)
    vs_o, adv_o, rho_o = L.vtrace(**tr, rho_bar=rb, c_bar=cb)
    vs = torch.empty(T, B, dtype=torch.float32, device="cuda")
    adv = torch.empty_like(vs)
    rho = torch.empty_like(vs)
    A.accerl_vtrace(_dev(tr["logits_original"]), _dev(tr["logits_smaller"]), _dev(tr["actions"]), _dev(tr["rewards"]),
                    _dev(tr["discounts"]), _dev(tr["values"]), _dev(tr["bootstrap"]), rb, cb, vs, adv, rho)
    torch.cuda.synchronize()
    scale = max(1.0, float(np.abs(vs_o).max()))
    assert np.allclose(rho.cpu().numpy(), rho_o, rtol=2e-5, atol=1e-6)
    assert np.allclose(vs.cpu().numpy(), vs_o, rtol=1e-4, atol=2e-5 * scale)
    assert np.allclose(adv.cpu().numpy(), adv_o, rtol=1e-4, atol=2e-5 * scale)
    # the advantage output is optional
    vs2 = torch.empty_like(vs)
    rho2 = torch.empty_like(vs)
    A.accerl_vtrace(_dev(tr["logits_original"]), _dev(tr["logits_smaller"]), _dev(tr["actions"]), _dev(tr["rewards"]),
                    _dev(tr["discounts"]), _dev(tr["values"]), _dev(tr["bootstrap"]), rb, cb, vs2, None, rho2)
    torch.cuda.synchronize()
    assert torch.equal(vs, vs2) and torch.equal(rho, rho2)


def test_vtrace_on_policy_returns(A):
    T, B, nA = 12, 130, 9
    tr = wl.make_trajectory(T, B, nA)
    tr["logits_smaller"] = tr["logits_original"].copy()
    vs = torch.empty(T, B, dtype=torch.float32, device="cuda")
    rho = torch.empty_like(vs)
    A.accerl_vtrace(_dev(tr["logits_original"]), _dev(tr["logits_smaller"]), _dev(tr["actions"]), _dev(tr["rewards"]),
                    _dev(tr["discounts"]), _dev(tr["values"]), _dev(tr["bootstrap"]), 1.0, 1.0, vs, None, rho)
    torch.cuda.synchronize()
    assert float((rho - 1).abs().max()) == 0.0
    want = np.empty((T, B))
    nxt = tr["bootstrap"].astype(np.float64)
    for t in range(T - 1, -1, -1):
        nxt = tr["rewards"][t] + tr["discounts"][t].astype(np.float64) * nxt
        want[t] = nxt
    assert np.allclose(vs.cpu().numpy(), want, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("B,nA,beta", [(1, 2, 0.0), (4096 + 5, 18, 0.01), (700, 64, 1.0)])
def test_distill_loss_matches_oracle(A, B, nA, beta):
    lo, ls = wl.make_logits_pair(B, nA, gap=0.5)
    vo = wl.normal(wl.BASE_SEED, 77, 0, B)
    vs = wl.normal(wl.BASE_SEED, 78, 0, B)
    loss_o, mean_o = L.distill_loss(lo, ls, vo, vs, beta)
    loss = torch.empty(B, dtype=torch.float32, device="cuda")
    mean = torch.zeros(1, dtype=torch.float64, device="cuda")
    A.accerl_distill_loss(_dev(lo), _dev(ls), _dev(vo), _dev(vs), beta, loss, mean)
    torch.cuda.synchronize()
    assert np.allclose(loss.cpu().numpy(), loss_o, rtol=1e-4, atol=1e-5)
    assert np.isclose(float(mean[0]), mean_o, rtol=1e-4, atol=1e-6)
    mean2 = torch.zeros(1, dtype=torch.float64, device="cuda")
    A.accerl_distill_loss(_dev(lo), _dev(ls), _dev(vo), _dev(vs), beta, None, mean2)
    torch.cuda.synchronize()
    assert float(mean2[0]) == float(mean[0])
