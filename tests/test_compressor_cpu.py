"""The package's own PTQ / pruning helper agrees with the oracle's (independent code, same reading)."""
import numpy as np

import oracle
import workloads as wl
from paper_2211_15023_amd import compressor
from helpers import make_states


def test_ptq_and_pruning_agree_with_oracle():
    for ci in (0, 3, 4):
        cfg = wl.CONFIGS[ci]
        nt, ns = cfg["teacher"], cfg["student"]
        pt = wl.init_params(nt, wl.STREAM["weights_teacher"])
        if cfg["student_from"] == "prune":
            ps_o, _ = oracle.prune_policy(nt, pt, ns)
            ps_c = compressor.prune_policy(nt, pt, ns)
            for (n1, w1, b1), (n2, w2, b2) in zip(ps_o, ps_c):
                assert n1 == n2 and np.array_equal(w1, w2)
                assert (b1 is None and b2 is None) or np.array_equal(b1, b2)
        else:
            ps_o = pt
        calib = make_states(ns, 24, wl.STREAM["calibration"])
        qp = oracle.quantize_policy(ns, ps_o, calib)
        tensors, scales = compressor.quantize_policy(ns, ps_o, calib)
        assert len(tensors) == len(qp.tensors)
        for a, b in zip(tensors, qp.tensors):
            assert set(a) - {"name"} == set(b) - {"name"}
            for k in ("wq", "s_w", "w"):
                if k in a:
                    assert np.array_equal(a[k], b[k]), (ci, a["name"], k)
        assert scales.shape == qp.act_scales.shape
        np.testing.assert_allclose(scales, qp.act_scales, rtol=2e-5)
