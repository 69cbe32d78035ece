"""Pins for the quantizer, the pruner and the whole-network walk of the oracle."""
import os

import numpy as np
import torch
import torch.nn.functional as F

import oracle
import workloads as wl
from oracle import layers as L
from oracle.ptq import quantize_weight, derived_constants
from helpers import policies, make_states, rel_err_rows

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(4242)


def _read_table(path):
    rows = []
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append(line.split())
    return rows


def test_paper_network_table_shapes():
    """Filter counts/sizes, input and output range of the paper's network table; strides 4/2/1 and
    no padding give 20 -> 9 -> 7 and a 3136-wide flatten for the original network."""
    rows = {r[0]: r for r in _read_table(os.path.join(GOLD, "paper_network_table.txt"))}

    def parse(tok):
        n, k = tok.rstrip(")").split("(")
        return int(n), int(k)

    org = wl.nature_cnn()
    convs = [l for l in org.layers if l["kind"] == "conv"]
    for l, tok in zip(convs, rows["Original"][4:7]):
        assert (l["cout"], l["k"]) == parse(tok)
    assert org.obs_shape == tuple(int(v) for v in rows["Original"][1:4]) and org.n_actions <= int(rows["Original"][8])
    shp = wl.trace_shapes(org)
    assert [s for s in shp[:4]] == [(32, 20, 20), (64, 9, 9), (64, 7, 7), (3136,)]
    assert (84 - 8) // 4 + 1 == 20 and (20 - 4) // 2 + 1 == 9 and 9 - 3 + 1 == 7 and 64 * 49 == 3136
    for name in ("Net1", "Net2", "Net3"):
        net = wl.configs.PAPER_STUDENTS[name.lower()]
        convs = [l for l in net.layers if l["kind"] == "conv"]
        assert len(convs) == 2 and rows[name][6] == "-"
        for l, tok in zip(convs, rows[name][4:6]):
            assert (l["cout"], l["k"]) == parse(tok)
        assert [l for l in net.layers if l["kind"] == "dense"][0]["cout"] == int(rows[name][7])
    imp = wl.trace_shapes(wl.impala_cnn("t"))
    assert imp[1] == (16, 42, 42) and imp[5] == (32, 21, 21) and imp[9] == (32, 11, 11) and imp[13] == (3872,)


def test_paper_timing_arithmetic():
    kv = {r[0]: float(r[1]) for r in _read_table(os.path.join(GOLD, "paper_timing.txt"))}
    collect = kv["n_steps"] * (kv["env_ms"] + kv["agent_ms"])
    assert collect == kv["collect_ms"]
    assert round(100 * collect / (collect + kv["learn_ms"]), 1) == kv["collect_share_pct"]
    assert round(100 * kv["n_steps"] * kv["agent_ms"] / (collect + kv["learn_ms"]), 1) == kv["agent_share_pct"]


def test_weight_quantization_properties():
    w = rng.standard_normal((6, 3, 4, 4)).astype(np.float32)
    w[2] = 0                                                    # an all-zero filter keeps scale 1
    q, s = quantize_weight(w)
    assert q.dtype == np.int8 and s.dtype == np.float32 and s[2] == 1.0 and not q[2].any()
    flat = np.abs(q.reshape(6, -1)).max(axis=1)
    assert np.all(flat[[0, 1, 3, 4, 5]] == 127) and np.abs(q).max() <= 127
    err = np.abs(w.astype(np.float64) - q.astype(np.float64) * s.astype(np.float64)[:, None, None, None])
    assert np.all(err.reshape(6, -1).max(axis=1) <= s.astype(np.float64) / 2 * (1 + 1e-6))
    # hand example: max 2.54 -> s = 0.02 ; 1.27 -> 63.5 -> tie to even 64 (double arithmetic: 63.4999.. or 63.5)
    q2, s2 = quantize_weight(np.array([[2.54, -2.54, 0.0, 0.02]], np.float32))
    assert q2.tolist() == [[127, -127, 0, 1]] and abs(s2[0] - 0.02) < 1e-8


def test_derived_constants_hand_example():
    net = wl.mlp("tiny", 2, (2,), 2)
    qp = oracle.QuantPolicy(
        tensors=[dict(name="l0.dense", wq=np.array([[127, 0], [0, -127]], np.int8), s_w=np.array([0.01, 0.02], np.float32),
                      b=np.array([0.5, -0.25], np.float32)),
                 dict(name="heads", wq=np.ones((3, 2), np.int8), s_w=np.array([0.1, 0.1, 0.2], np.float32),
                      b=np.array([1.0, 0.0, -1.0], np.float32))],
        act_scales=np.array([0.5, 0.25], np.float32))
    dc = derived_constants(net, qp)
    assert dc["inv_s0"] == np.float32(2.0)
    s_w = np.array([0.01, 0.02], np.float32).astype(np.float64)
    assert dc["layers"][0]["biasq"].tolist() == [int(np.rint(0.5 / (0.5 * s_w[0]))), int(np.rint(-0.25 / (0.5 * s_w[1])))]
    assert dc["layers"][0]["biasq"].tolist() == [100, -25]
    np.testing.assert_array_equal(dc["layers"][0]["m"], ((0.5 * s_w) / 0.25).astype(np.float32))
    s_h = np.array([0.1, 0.1, 0.2], np.float32).astype(np.float64)
    np.testing.assert_array_equal(dc["heads"]["d"], (0.25 * s_h).astype(np.float32))
    assert dc["heads"]["biasq"].tolist() == [40, 0, -20]
    # forward by hand: x = [1.0, -0.5] -> q = [2, -1]; acc = [254+100, 127-25]; *m=[.02,.04] -> 7.08, 4.08 -> [7, 4]
    out = oracle.forward_int8(net, qp, np.array([[1.0, -0.5]], np.float32), np.array([0.0], np.float32))
    # heads: acc = 11 + biasq -> [51, 11, -9]; logits = acc * d = 51*.025, 11*.025 ; value = -9*.05
    np.testing.assert_allclose(out["logits"], [[51 * 0.025, 11 * 0.025]], rtol=1e-6)
    np.testing.assert_allclose(out["value"], [-9 * 0.05], rtol=1e-6)


def test_float_network_vs_library_ops():
    """The teacher walk of the IMPALA net (conv, ignore-pad maxpool, residual blocks, flatten order,
    FC, heads) against the same graph written with library ops in float64."""
    net = wl.impala_cnn("t", (4, 6, 6), n_actions=5, fc=32)
    params = wl.init_params(net, 11)
    x8 = wl.make_frames_u8(3, stream=91)
    got = oracle.forward_float(net, params, x8, None, "fp32")
    P = {n: (torch.from_numpy(w).double(), None if b is None else torch.from_numpy(b).double()) for n, w, b in params}
    x = torch.from_numpy(x8).double() / 255.0
    for i, ly in enumerate(net.layers):
        kd = ly["kind"]
        if kd == "conv":
            x = F.conv2d(x, *P[f"l{i}.conv"], stride=ly["stride"], padding=ly["pad"])
            x = x.clamp_min(0) if ly["relu"] else x
        elif kd == "maxpool":
            x = F.max_pool2d(x, 3, 2, 1)
        elif kd == "resblock":
            t = F.conv2d(x.clamp_min(0), *P[f"l{i}.convA"], padding=1).clamp_min(0)
            x = x + F.conv2d(t, *P[f"l{i}.convB"], padding=1)
        elif kd == "relu":
            x = x.clamp_min(0)
        elif kd == "flatten":
            x = x.flatten(1)
        elif kd == "dense":
            x = F.linear(x, *P[f"l{i}.dense"]).clamp_min(0)
    out = F.linear(x, *P["heads"]).numpy()
    assert rel_err_rows(got["logits"], out[:, :5]).max() < 1e-5
    assert rel_err_rows(got["value"], out[:, 5]).max() < 1e-5


def test_pruning_is_row_column_deletion():
    """Section 2.2 (Structured Pruning): deleting feature maps equals deleting rows and columns of the
    parameter matrices, so the pruned fp32 student equals the teacher with those channels zeroed."""
    nt = wl.impala_cnn("t", (8, 12, 12), n_actions=6, fc=64)
    ns = wl.impala_cnn("s", (4, 6, 6), n_actions=6, fc=64)
    pt = wl.init_params(nt, 21)
    ps, kept = oracle.prune_policy(nt, pt, ns)
    assert [w.shape for _, w, _ in ps] == [tuple(s) for _, s, _ in wl.param_shapes(ns)]
    zeroed = []
    for name, w, b in pt:
        w, b = w.copy(), None if b is None else b.copy()
        if name in kept:
            drop = np.setdiff1d(np.arange(w.shape[0]), kept[name])
            w[drop] = 0
            b[drop] = 0
        zeroed.append((name, w, b))
    x = wl.make_frames_u8(4, stream=92)
    u = wl.make_uniforms(4)
    a = oracle.forward_float(ns, ps, x, u, "fp32")
    b = oracle.forward_float(nt, zeroed, x, u, "fp32")
    assert np.array_equal(a["logits"], b["logits"]) and np.array_equal(a["value"], b["value"])
    assert np.array_equal(a["action"], b["action"])
    # the kept set maximises the summed L1 norm over the stream's writers
    for name, keep in kept.items():
        if name.endswith("convA"):
            w = dict((n, w) for n, w, _ in pt)[name]
            l1 = np.abs(w).reshape(w.shape[0], -1).sum(1)
            assert set(keep) == set(np.argsort(-l1, kind="stable")[:len(keep)])


def test_int8_network_taps_are_consistent():
    """Every tap of the int8 walk is reproduced from the previous one by library integer ops."""
    nt, pt, ns, ps, qp = policies(3, 16)
    x = make_states(ns, 2, wl.STREAM["states"])
    taps = {}
    out = oracle.forward_int8(ns, qp, x, wl.make_uniforms(2), taps=taps)
    dc = derived_constants(ns, qp)
    # first conv: uint8 observations enter as 0..255 integers
    k0 = dc["layers"][0]
    ref = F.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(k0["wq"].astype(np.float64)),
                   torch.from_numpy(k0["biasq"].astype(np.float64)), padding=1).numpy()
    assert np.array_equal(taps[(0, "acc")], ref.astype(np.int64))
    # a residual block, from its input stream tap
    xin = taps[(1, "act")]
    k2 = dc["layers"][2]
    accA = F.conv2d(torch.from_numpy(np.maximum(xin, 0).astype(np.float64)), torch.from_numpy(k2["wqA"].astype(np.float64)),
                    torch.from_numpy(k2["biasqA"].astype(np.float64)), padding=1).numpy()
    assert np.array_equal(taps[(2, "accA")], accA.astype(np.int64))
    actA = np.clip(np.rint(taps[(2, "accA")].astype(np.float32) * k2["mA"].reshape(1, -1, 1, 1)), 0, 127)
    assert np.array_equal(taps[(2, "actA")], actA.astype(np.int8))
    # flatten is C,H,W order and the last ReLU is applied on load by the FC
    i_fc = max(i for i, l in enumerate(ns.layers) if l["kind"] == "dense")
    last = taps[(i_fc - 3, "act")]
    kf = dc["layers"][i_fc]
    acc = np.maximum(last, 0).reshape(2, -1).astype(np.int64) @ kf["wq"].astype(np.int64).T + kf["biasq"]
    assert np.array_equal(taps[(i_fc, "acc")], acc)
    assert out["logits"].shape == (2, 18) and out["action"].shape == (2,)


def test_int8_student_tracks_fp32_network():
    """Loose sanity bound: on calibration-like states the int8 logits stay within a few percent of
    the fp32 logits of the same weights (propagated s/2 rounding errors)."""
    for ci, tol in ((0, 0.05), (1, 0.05), (2, 0.08), (3, 0.12)):
        nt, pt, ns, ps, qp = policies(ci, 64 if ci >= 2 else 256)
        x = make_states(ns, 32, wl.STREAM["states"])
        f = oracle.forward_float(ns, ps, x, None, "fp32")
        q = oracle.forward_int8(ns, qp, x, None)
        scale = np.abs(f["logits"]).max()
        assert np.median(np.abs(q["logits"] - f["logits"]).max(axis=1)) / scale < tol, ci
        b = oracle.forward_float(ns, ps, x, None, "bf16")
        assert np.abs(b["logits"] - f["logits"]).max() / scale < 3e-2, ci


def test_recurrent_network_walk():
    nt, pt, ns, ps, qp = policies(4, 16)
    B = 3
    x = make_states(ns, B, wl.STREAM["states"])
    h, c = wl.make_hc(B, 256)
    done = np.array([0, 1, 0], np.uint8)
    r = oracle.forward_int8(ns, qp, x, wl.make_uniforms(B), h=h, c=c, done=done)
    assert r["h"].shape == (B, 256) and np.isfinite(r["logits"]).all()
    # row 1 was reset: same as starting from zeros
    r0 = oracle.forward_int8(ns, qp, x, wl.make_uniforms(B), h=np.zeros_like(h), c=np.zeros_like(c))
    assert np.array_equal(r["h"][1], r0["h"][1]) and np.array_equal(r["logits"][1], r0["logits"][1])
    assert not np.array_equal(r["h"][0], r0["h"][0])
    # inputs are not modified
    h2, _ = wl.make_hc(B, 256)
    assert np.array_equal(h, h2)
    t = oracle.forward_float(nt, pt, x, None, "bf16", h=h, c=c, done=done)
    assert t["h"].shape == (B, 256)


def test_generators_are_counter_based():
    a = wl.make_frames_u8(8, first=0)
    b = wl.make_frames_u8(3, first=5)
    assert np.array_equal(a[5:8], b)
    assert np.array_equal(wl.make_obs_f32(10, 24)[4:7], wl.make_obs_f32(3, 24, first=4))
    assert np.array_equal(wl.make_uniforms(10)[6:], wl.make_uniforms(4, first=6))
    u = wl.make_uniforms(100000)
    assert u.min() >= 0 and u.max() < 1 and abs(u.mean() - 0.5) < 5e-3
    f = wl.make_frames_u8(16)
    # rectangles leave flat regions: many horizontally equal neighbours, unlike pure noise
    assert (f[..., 1:] == f[..., :-1]).mean() > 0.2


def test_recurrent_handoff_hand_example():
    """int8 torso -> bf16 recurrent core: the FC's int8 output is dequantized by the FC's own output scale
    (the last activation scale), and the cell reads that vector.  A two-unit FC in front of a one-unit LSTM
    whose only live input path is the candidate gate g, with i and o held open by their biases: everything
    is a closed form of the two dequantized features."""
    net = wl.Net("tiny_rec", "f32", (2,), 2, [wl.dense(2, 2, True), wl.lstm(2, 1)])
    w_ih = np.zeros((4, 2), np.float32)
    w_ih[2] = [1.0, 2.0]                                   # gate order i, f, g, o
    bias = np.array([20.0, 0.0, 0.0, 20.0], np.float32)
    qp = oracle.QuantPolicy(
        tensors=[dict(name="l0.dense", wq=np.array([[127, 0], [0, 64]], np.int8), s_w=np.array([0.01, 0.02], np.float32),
                      b=np.zeros(2, np.float32)),
                 dict(name="l1.lstm_ih", w=w_ih, b=bias),
                 dict(name="l1.lstm_hh", w=np.zeros((4, 1), np.float32), b=None),
                 dict(name="heads", w=np.array([[1.0], [-1.0], [0.5]], np.float32), b=np.array([0.0, 0.25, 1.0], np.float32))],
        act_scales=np.array([0.5, 0.25], np.float32))
    # x = [1.0, 0.5] -> q = [2, 1]; acc = [254, 64]; m = 0.5 * s_w / 0.25 = [.02, .04] -> 5.08, 2.56 -> [5, 3]
    # dequantized with the FC's output scale 0.25: [1.25, 0.75] (0.5 or a weight scale would give other values)
    x = np.array([[1.0, 0.5]], np.float32)
    taps = {}
    r = oracle.forward_int8(net, qp, x, np.array([0.0], np.float32), h=np.zeros((1, 1), np.float32),
                            c=np.zeros((1, 1), np.float32), taps=taps)
    assert taps[(0, "act")].tolist() == [[5, 3]]
    sig = lambda v: 1.0 / (1.0 + np.exp(-v))
    g = 1.0 * 1.25 + 2.0 * 0.75
    c_ref = sig(0.0) * 0.0 + sig(20.0) * np.tanh(g)
    h_ref = sig(20.0) * np.tanh(c_ref)
    assert abs(float(r["c"][0, 0]) - c_ref) < 1e-6 and abs(float(r["h"][0, 0]) - h_ref) < 1e-6
    # the heads read bf16(h'): one rounding of 2^-9 relative at most
    hb = float(L.bf16_round(r["h"])[0, 0])
    assert abs(hb - h_ref) <= abs(h_ref) * 2.0 ** -8
    np.testing.assert_allclose(r["logits"], [[hb, -hb + 0.25]], rtol=1e-6)
    np.testing.assert_allclose(r["value"], [0.5 * hb + 1.0], rtol=1e-6)
    # a carried state enters through the forget gate (sigma(0) = 1/2) and is wiped by done
    r2 = oracle.forward_int8(net, qp, x, None, h=np.full((1, 1), 0.3, np.float32), c=np.full((1, 1), 0.8, np.float32))
    assert abs(float(r2["c"][0, 0]) - (0.5 * 0.8 + sig(20.0) * np.tanh(g))) < 1e-6
    r3 = oracle.forward_int8(net, qp, x, None, h=np.full((1, 1), 0.3, np.float32), c=np.full((1, 1), 0.8, np.float32),
                             done=np.array([1], np.uint8))
    assert np.array_equal(r3["c"], r["c"]) and np.array_equal(r3["h"], r["h"])


def test_mixture_rows_equal_each_networks_own_forward():
    """Section 3.2 mixture: a row holds exactly what the chosen network alone produces for it."""
    nt, pt, ns, ps, qp = policies(1)
    B = 23
    x = make_states(ns, B, wl.STREAM["states"])
    u = wl.make_uniforms(B)
    own_s = oracle.forward_int8(ns, qp, x, u)
    own_t = oracle.forward_float(nt, pt, x, u, "fp32")
    flags = (rng.random(B) < 0.4).astype(np.uint8)
    assert flags.any() and not flags.all()
    for use in (flags, np.ones(B, np.uint8), np.zeros(B, np.uint8)):
        mix = oracle.forward_mixture(ns, qp, nt, pt, "fp32", x, u, use)
        sel = use.astype(bool)
        for k in ("logits", "value", "action"):
            assert np.array_equal(mix[k][sel], own_s[k][sel]), k
            assert np.array_equal(mix[k][~sel], own_t[k][~sel]), k
