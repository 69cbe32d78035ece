"""The entry point that allocates nothing (accerl_monitor_kl_noalloc) against accerl_monitor_kl, through the C ABI.

Two calls in a row on the library's one fixed partial-sum array, the second on a smaller input: per-row KL and entropy
must be identical to the allocating entry point's (same kernels), the fp64 statistics identical whenever both passes use
the same number of workgroups (up to 262 144 rows) and equal to 1e-12 relative beyond; both are also held to the fp64
oracle with the bounds of test_gpu_monitor.py.  Sizes beyond the stated maximum are rejected before anything is enqueued.
"""
import ctypes as C

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


def _both(A, B, nA, first):
    lo, ls = wl.make_logits_pair(B, nA, gap=0.5, first=first)
    dlo, dls = _dev(lo), _dev(ls)
    res = []
    for fn in (A.accerl_monitor_kl_noalloc, A.accerl_monitor_kl):
        kl = torch.full((B,), -7.0, dtype=torch.float32, device="cuda")
        ent = torch.full((B,), -7.0, dtype=torch.float32, device="cuda")
        st = torch.full((4,), -7.0, dtype=torch.float64, device="cuda")
        fn(dlo, dls, kl, ent, st)
        torch.cuda.synchronize()
        res.append((kl.cpu().numpy(), ent.cpu().numpy(), st.cpu().numpy()))
    return lo, ls, res


# first a long input (every record of the fixed array written), then shorter ones that use a part of it
@pytest.mark.parametrize("sizes", [((300000, 18), (4096 + 17, 18), (63, 18)), ((1000, 64), (1, 2))])
def test_noalloc_matches_allocating_entry_point(A, sizes):
    first = 0
    for B, nA in sizes:
        print(f"monitor no-alloc B={B} A={nA}", flush=True)
        lo, ls, ((kl_n, ent_n, st_n), (kl_a, ent_a, st_a)) = _both(A, B, nA, first)
        first += B
        assert np.array_equal(kl_n, kl_a) and np.array_equal(ent_n, ent_a)
        if B <= 1024 * 256:
            assert np.array_equal(st_n, st_a)
        else:
            assert np.allclose(st_n, st_a, rtol=1e-12, atol=0)
        kl_o, ent_o, st_o = L.kl_monitor(lo, ls)
        assert np.allclose(kl_n, kl_o, rtol=2e-4, atol=3e-6) and np.allclose(ent_n, ent_o, rtol=2e-5, atol=3e-6)
        assert np.isclose(st_n[0], st_o[0], rtol=1e-4, atol=1e-6) and np.isclose(st_n[1], st_o[1], rtol=2e-4, atol=3e-6)
        assert np.isclose(st_n[2], st_o[2], rtol=1e-3, atol=1e-7) and np.isclose(st_n[3], st_o[3], rtol=1e-5)


def test_noalloc_rejects_oversize_and_bad_arguments(A):
    lib = A.load_library()
    x = torch.zeros(64, 18, dtype=torch.float32, device="cuda")
    st = torch.zeros(4, dtype=torch.float64, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())
    # more rows than the fixed array is specified for: refused from the size alone, nothing is read
    assert lib.accerl_monitor_kl_noalloc(p(x), p(x), (1 << 24) + 1, 18, None, None, p(st), None) == -1
    assert "exceed" in A.accerl_last_error()
    assert lib.accerl_monitor_kl_noalloc(p(x), p(x), 64, 65, None, None, p(st), None) == -1
    assert lib.accerl_monitor_kl_noalloc(None, p(x), 64, 18, None, None, p(st), None) == -1
    assert lib.accerl_monitor_kl_noalloc(p(x), p(x), 0, 18, None, None, p(st), None) == 0
    torch.cuda.synchronize()
    assert st.cpu().numpy().tolist() == [0.0] * 4
