"""The actor forward pass as a walk over a layer list, one oracle layer call per step.

forward_float : the teacher: fp32, or bf16 (GEMM operands and every stored layer output --
                conv, FC, residual sum -- rounded to bfloat16; accumulation, bias, ReLU, pooling
                and the LSTM gate arithmetic in fp32; h, c and the head outputs stay fp32).
forward_int8  : the post-training-quantized student (paper Section 2.2, "Parameter
                Quantization": int8 parameters, Conv/FC+ReLU fused; arithmetic as stated in
                oracle.c).
Both return logits [B,A], value [B], action [B] and, on request, every intermediate tensor.
"""
import numpy as np

from . import layers as L


def _params_iter(params):
    return iter(params)


def _heads_out(net, out, u):
    A = net.n_actions
    logits = np.ascontiguousarray(out[:, :A])
    value = np.ascontiguousarray(out[:, A])
    action = L.softmax_sample(logits, u) if u is not None else None
    return logits, value, action


def forward_float(net, params, states, uniforms=None, precision="fp32", h=None, c=None, done=None,
                  observe=None):
    """params: list of (name, W, b) fp32 in blob order.  precision: "fp32" or "bf16".

    observe(tag, array), if given, is called on the input and on every tensor that the int8
    student stores quantized (used by calibration).  Returns a dict.
    """
    bf = precision == "bf16"
    assert precision in ("fp32", "bf16")
    it = _params_iter(params)
    if net.obs_dtype == "u8":
        assert states.dtype == np.uint8
        x = states.astype(np.float32) / np.float32(255.0)      # one fp32 division per pixel
    else:
        x = np.ascontiguousarray(states, dtype=np.float32)
    obs = observe or (lambda tag, a: None)
    obs("input", x)
    for i, ly in enumerate(net.layers):
        kd = ly["kind"]
        if kd == "conv":
            _, w, b = next(it)
            x = L.conv2d_f(x, w, b, ly["stride"], ly["pad"], ly["relu"], bf)
            x = L.bf16_round(x) if bf else x
            obs((i, "out"), x)
        elif kd == "dense":
            _, w, b = next(it)
            x = L.dense_f(x, w, b, ly["relu"], bf)
            x = L.bf16_round(x) if bf else x
            obs((i, "out"), x)
        elif kd == "maxpool":
            x = L.maxpool_f(x, ly["k"], ly["stride"], ly["pad"])
        elif kd == "resblock":
            _, wa, ba = next(it)
            _, wb, bb = next(it)
            a = np.maximum(x, np.float32(0))
            a = L.conv2d_f(a, wa, ba, 1, 1, True, bf)
            a = L.bf16_round(a) if bf else a
            obs((i, "mid"), a)
            t = L.conv2d_f(a, wb, bb, 1, 1, False, bf)
            x = x + t                                              # fp32 add of the unrounded branch
            x = L.bf16_round(x) if bf else x
            obs((i, "out"), x)
        elif kd == "relu":
            x = np.maximum(x, np.float32(0))
        elif kd == "flatten":
            x = np.ascontiguousarray(x.reshape(x.shape[0], -1))
        elif kd == "lstm":
            _, wih, bias = next(it)
            _, whh, _ = next(it)
            B = x.shape[0]
            if h is None:
                h = np.zeros((B, ly["hidden"]), np.float32)
                c = np.zeros((B, ly["hidden"]), np.float32)
            h, c = L.lstm_step(x, h, c, done, wih, whh, bias, bf)
            x = h
        else:
            raise ValueError(kd)
    _, wh, bh = next(it)
    out = L.dense_f(x, wh, bh, False, bf)
    logits, value, action = _heads_out(net, out, uniforms)
    return dict(logits=logits, value=value, action=action, h=h, c=c, features=x)


def forward_int8(net, qp, states, uniforms=None, h=None, c=None, done=None, taps=None):
    """qp: ptq.QuantPolicy.  taps: optional dict filled with {(layer, tag): array} for the
    int32 accumulators ("acc", "accA", "accB") and int8 outputs ("act", "actA") of each layer,
    all in logical NCHW / [B, features] order."""
    from .ptq import derived_constants
    dc = derived_constants(net, qp)
    tp = taps if taps is not None else {}
    if net.obs_dtype == "u8":
        assert states.dtype == np.uint8
        xq = np.ascontiguousarray(states)                 # 0..255, scale 1/255, no zero point
    else:
        xq = L.quantize_f32(states, dc["inv_s0"])
        tp[(-1, "act")] = xq
    relu_in = False
    float_x = None
    for i, ly in enumerate(net.layers):
        kd = ly["kind"]
        k = dc["layers"].get(i)
        if kd == "conv":
            acc = L.conv2d_q_acc(xq, k["wq"], k["biasq"], ly["stride"], ly["pad"], relu_in)
            xq = L.requant(acc, k["m"], 0 if ly["relu"] else -127)
            tp[(i, "acc")], tp[(i, "act")] = acc, xq
            relu_in = False
        elif kd == "dense":
            acc = L.dense_q_acc(xq, k["wq"], k["biasq"], relu_in)
            xq = L.requant(acc, k["m"], 0 if ly["relu"] else -127)
            tp[(i, "acc")], tp[(i, "act")] = acc, xq
            relu_in = False
        elif kd == "maxpool":
            assert not relu_in
            xq = L.maxpool_i8(xq, ly["k"], ly["stride"], ly["pad"])
            tp[(i, "act")] = xq
        elif kd == "resblock":
            assert not relu_in
            acca = L.conv2d_q_acc(xq, k["wqA"], k["biasqA"], 1, 1, True)
            aq = L.requant(acca, k["mA"], 0)
            accb = L.conv2d_q_acc(aq, k["wqB"], k["biasqB"], 1, 1, False)
            xq = L.requant_residual(accb, xq, k["r"], k["mB"])
            tp[(i, "accA")], tp[(i, "actA")], tp[(i, "accB")], tp[(i, "act")] = acca, aq, accb, xq
        elif kd == "relu":
            relu_in = True                                 # applied by the next consumer's load
        elif kd == "flatten":
            xq = np.ascontiguousarray(xq.reshape(xq.shape[0], -1))
        elif kd == "lstm":
            if relu_in:
                xq = np.maximum(xq, 0).astype(np.int8)
                relu_in = False
            x = L.dequant_i8(xq, k["s_in"])
            B = x.shape[0]
            if h is None:
                h = np.zeros((B, ly["hidden"]), np.float32)
                c = np.zeros((B, ly["hidden"]), np.float32)
            h, c = L.lstm_step(x, h, c, done, k["w_ih"], k["w_hh"], k["bias"], True)
            float_x = h
        else:
            raise ValueError(kd)
    hd = dc["heads"]
    if float_x is not None:                                # heads after a bf16 recurrent core
        out = L.dense_f(float_x, hd["w"], hd["b"], False, True)
    else:
        acc = L.dense_q_acc(xq, hd["wq"], hd["biasq"], relu_in)
        tp[("heads", "acc")] = acc
        out = L.dequant(acc, hd["d"])
    logits, value, action = _heads_out(net, out, uniforms)
    return dict(logits=logits, value=value, action=action, h=h, c=c)


def forward_mixture(net_small, qp_small, net_orig, params_orig, precision_orig, states, uniforms, use_smaller):
    """alpha-mixture of Section 3.2 ("Knowledge Distillation Results"): row b goes through the int8 smaller
    network where use_smaller[b] is set, else through the original network; rows are independent, so the
    result is each network's own output on its rows."""
    use = np.asarray(use_smaller).astype(bool)
    B = len(use)
    A = net_small.n_actions
    out = dict(logits=np.zeros((B, A), np.float32), value=np.zeros(B, np.float32), action=np.zeros(B, np.int32))
    if use.any():
        r = forward_int8(net_small, qp_small, states[use], uniforms[use])
        for k in out:
            out[k][use] = r[k]
    if (~use).any():
        r = forward_float(net_orig, params_orig, states[~use], uniforms[~use], precision_orig)
        for k in out:
            out[k][~use] = r[k]
    return out
