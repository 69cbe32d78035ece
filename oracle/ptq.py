"""Post-training quantization and structured pruning: fp32 weights -> student policy.

Paper Section 2.2: "Parameter Quantization" replaces fp32 parameters by int8 after training
(no retraining); "Structured Pruning" deletes whole feature maps / neurons, i.e. rows and
columns of the weight matrices.  The paper fixes neither scales nor rounding; the reading:

  weights      per output channel n: s_w[n] = max|W[n,:]| / 127 (1 if zero),
               Wq = clamp(rint(W / s_w[n]), -127, 127), computed in double
  activations  per tensor, symmetric: s_a = max|a| / 127 over the calibration states run
               through the fp32 network (1 if zero); uint8 observations are the exception:
               they keep their 0..255 integers with scale 1/255
  bias         biasq[n] = rint(b[n] / (s_in * s_w[n])) as int32 (double arithmetic)
  requant      m[n] = float((double)s_in * s_w[n] / s_out); residual ratio r = float(s_x / s_out);
               head dequant d[n] = float((double)s_in * s_w[n]); input inv_s0 = float(1 / s_0)
  pruning      keep the channels with the largest filter L1 norm (ties: lower index); all
               convolutions that write one residual stream share one kept set, ranked by the
               sum of their L1 norms; the hidden FC layer is kept whole
"""
from dataclasses import dataclass, field
from typing import List

import numpy as np

from workloads import trace_shapes

from .forward import forward_float


@dataclass
class QuantPolicy:
    """tensors: per parametrised tensor in blob order a dict with name, and either
    wq (int8) + s_w (float32 [out]) + b (float32) for quantized tensors or w + b (float32)
    for tensors that stay in float (recurrent core, heads behind it).
    act_scales: float32, s_0 first, then one per quantized activation tensor in layer order
    (conv/dense: its output; resblock: after conv A, then the stream after the add)."""
    tensors: List[dict] = field(default_factory=list)
    act_scales: np.ndarray = None


def quantize_weight(w):
    w = np.asarray(w, np.float64)
    flat = w.reshape(w.shape[0], -1)
    mx = np.abs(flat).max(axis=1)
    s = np.where(mx > 0, mx / 127.0, 1.0).astype(np.float32)
    q = np.clip(np.rint(flat / s.astype(np.float64)[:, None]), -127, 127).astype(np.int8)
    return q.reshape(w.shape), s


def _scale_from_maxabs(mx):
    return np.float32(mx / 127.0) if mx > 0 else np.float32(1.0)


def quantize_policy(net, params, calib_states):
    """params: [(name, W, b)] fp32.  Returns a QuantPolicy for `net`."""
    seen = {}

    def observe(tag, a):
        seen[tag] = float(np.abs(a.astype(np.float64)).max())

    forward_float(net, params, calib_states, None, "fp32", observe=observe)
    scales = [np.float32(1.0 / 255.0) if net.obs_dtype == "u8" else _scale_from_maxabs(seen["input"])]
    has_lstm = False
    for i, ly in enumerate(net.layers):
        if ly["kind"] in ("conv", "dense"):
            scales.append(_scale_from_maxabs(seen[(i, "out")]))
        elif ly["kind"] == "resblock":
            scales.append(_scale_from_maxabs(seen[(i, "mid")]))
            scales.append(_scale_from_maxabs(seen[(i, "out")]))
        elif ly["kind"] == "lstm":
            has_lstm = True
    tensors = []
    for name, w, b in params:
        if "lstm" in name or (name == "heads" and has_lstm):
            tensors.append(dict(name=name, w=np.asarray(w, np.float32), b=None if b is None else np.asarray(b, np.float32)))
        else:
            q, s = quantize_weight(w)
            tensors.append(dict(name=name, wq=q, s_w=s, b=np.asarray(b, np.float32)))
    return QuantPolicy(tensors=tensors, act_scales=np.asarray(scales, np.float32))


def _biasq(b, s_in, s_w):
    return np.rint(b.astype(np.float64) / (np.float64(s_in) * s_w.astype(np.float64))).astype(np.int32)


def _mult(s_in, s_w, s_out):
    return ((np.float64(s_in) * s_w.astype(np.float64)) / np.float64(s_out)).astype(np.float32)


def derived_constants(net, qp):
    """Integer biases and fp32 multipliers of every layer, from the scales (see module doc)."""
    sc = iter(qp.act_scales)
    tn = iter(qp.tensors)
    s_cur = np.float32(next(sc))
    out = dict(inv_s0=np.float32(1.0 / np.float64(s_cur)), layers={})
    for i, ly in enumerate(net.layers):
        kd = ly["kind"]
        if kd in ("conv", "dense"):
            t = next(tn)
            s_out = np.float32(next(sc))
            out["layers"][i] = dict(wq=t["wq"], biasq=_biasq(t["b"], s_cur, t["s_w"]),
                                    m=_mult(s_cur, t["s_w"], s_out))
            s_cur = s_out
        elif kd == "resblock":
            ta, tb = next(tn), next(tn)
            s1, s_out = np.float32(next(sc)), np.float32(next(sc))
            out["layers"][i] = dict(
                wqA=ta["wq"], biasqA=_biasq(ta["b"], s_cur, ta["s_w"]), mA=_mult(s_cur, ta["s_w"], s1),
                wqB=tb["wq"], biasqB=_biasq(tb["b"], s1, tb["s_w"]), mB=_mult(s1, tb["s_w"], s_out),
                r=np.float32(np.float64(s_cur) / np.float64(s_out)))
            s_cur = s_out
        elif kd == "lstm":
            tih, thh = next(tn), next(tn)
            out["layers"][i] = dict(s_in=s_cur, w_ih=tih["w"], w_hh=thh["w"], bias=tih["b"])
            s_cur = None
    t = next(tn)
    if "wq" in t:
        out["heads"] = dict(wq=t["wq"], biasq=_biasq(t["b"], s_cur, t["s_w"]),
                            d=(np.float64(s_cur) * t["s_w"].astype(np.float64)).astype(np.float32))
    else:
        out["heads"] = dict(w=t["w"], b=t["b"])
    return out


# ------------------------------------------------------------------ structured pruning

def _keep(l1, n_keep):
    order = np.lexsort((np.arange(l1.size), -l1))      # descending L1, ties: lower index first
    return np.sort(order[:n_keep])


def prune_policy(net_t, params_t, net_s):
    """Delete channels of teacher `params_t` (for net_t) to reach the widths of net_s.

    Returns (params_s, kept) where kept maps tensor name -> kept output-channel indices.
    Both nets must have the same layer kinds in the same order.
    """
    assert [l["kind"] for l in net_t.layers] == [l["kind"] for l in net_s.layers]
    P = {n: (np.asarray(w, np.float32), None if b is None else np.asarray(b, np.float32)) for n, w, b in params_t}
    l1 = lambda w: np.abs(w.astype(np.float64)).reshape(w.shape[0], -1).sum(axis=1)
    new, kept = {}, {}
    cur_keep = None            # kept indices of the tensor feeding the next layer (None = all)
    cur_hw = None              # spatial size per channel when a flatten follows
    shapes_t = trace_shapes(net_t)
    i = 0
    layers_t, layers_s = net_t.layers, net_s.layers
    while i < len(layers_t):
        lt, ls = layers_t[i], layers_s[i]
        kd = lt["kind"]
        if kd == "conv":
            # the stream this conv writes is also written by the convB of directly following resblocks
            writers = [f"l{i}.conv"]
            j = i + 1
            while j < len(layers_t) and layers_t[j]["kind"] in ("maxpool", "resblock", "relu"):
                if layers_t[j]["kind"] == "resblock":
                    writers.append(f"l{j}.convB")
                j += 1
            score = sum(l1(P[n][0]) for n in writers)
            keep = _keep(score, ls["cout"])
            for n in writers:
                kept[n] = keep
            w, b = P[f"l{i}.conv"]
            w = w if cur_keep is None else w[:, cur_keep]
            new[f"l{i}.conv"] = (w[keep], b[keep])
            cur_keep = keep
        elif kd == "resblock":
            wa, ba = P[f"l{i}.convA"]
            wb, bb = P[f"l{i}.convB"]
            keep_mid = _keep(l1(wa), ls["ch"])
            kept[f"l{i}.convA"] = keep_mid
            new[f"l{i}.convA"] = (wa[keep_mid][:, cur_keep], ba[keep_mid])
            new[f"l{i}.convB"] = (wb[cur_keep][:, keep_mid], bb[cur_keep])
        elif kd == "flatten":
            hw = int(np.prod(shapes_t[i - 1][1:])) if i > 0 else int(np.prod(net_t.obs_shape[1:]))
            if cur_keep is not None:
                cur_keep = (cur_keep[:, None] * hw + np.arange(hw)[None, :]).reshape(-1)
        elif kd == "dense":
            w, b = P[f"l{i}.dense"]
            assert ls["cout"] == lt["cout"], "hidden FC layers are kept whole"
            new[f"l{i}.dense"] = (w if cur_keep is None else w[:, cur_keep], b)
            cur_keep = None
        elif kd == "lstm":
            assert cur_keep is None
            new[f"l{i}.lstm_ih"] = P[f"l{i}.lstm_ih"]
            new[f"l{i}.lstm_hh"] = P[f"l{i}.lstm_hh"]
        i += 1
    w, b = P["heads"]
    new["heads"] = (w if cur_keep is None else w[:, cur_keep], b)
    params_s = [(n, np.ascontiguousarray(new[n][0]), None if new[n][1] is None else np.ascontiguousarray(new[n][1]))
                for n, _, _ in params_t]
    return params_s, kept
