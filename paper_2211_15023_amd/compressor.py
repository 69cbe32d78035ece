"""Host-side Compressor output for the actor library: post-training quantization and channel pruning.

Paper Section 2.2: the Compressor turns the Learner's fp32 network into the Actor's network
("Parameter Quantization": PTQ to int8; "Structured Pruning": delete feature maps, i.e. rows and
columns of the weight matrices).  This module produces exactly the two blobs accerl_policy_create
takes -- int8 weights with per-output-channel scales, and per-tensor activation scales from a
calibration batch -- using plain PyTorch CPU ops for the calibration pass.  It runs once per policy,
off the hot path; the forward itself never leaves the HIP kernels.
"""
import numpy as np
import torch
import torch.nn.functional as F


def quantize_weight(w):
    """s_w[n] = max|W[n]| / 127 (1 for an all-zero row); Wq = clamp(rint(W / s_w), -127, 127)."""
    w64 = np.asarray(w, np.float64)
    flat = w64.reshape(w64.shape[0], -1)
    mx = np.abs(flat).max(axis=1)
    s = np.where(mx > 0, mx / 127.0, 1.0).astype(np.float32)
    q = np.clip(np.rint(flat / s.astype(np.float64)[:, None]), -127, 127).astype(np.int8)
    return q.reshape(w64.shape), s


def _scale(t):
    mx = float(t.abs().max())
    return np.float32(mx / 127.0) if mx > 0 else np.float32(1.0)


@torch.no_grad()
def calibrate(net, params, calib_states):
    """Activation scales (s_0 first) from an fp32 pass over the calibration states."""
    P = iter(params)
    if net.obs_dtype == "u8":
        x = torch.from_numpy(np.ascontiguousarray(calib_states)).float() / 255.0
        scales = [np.float32(1.0 / 255.0)]
    else:
        x = torch.from_numpy(np.ascontiguousarray(calib_states, dtype=np.float32))
        scales = [_scale(x)]
    tt = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    for L in net.layers:
        kd = L["kind"]
        if kd == "conv":
            _, w, b = next(P)
            x = F.conv2d(x, tt(w), tt(b), stride=L["stride"], padding=L["pad"])
            x = x.clamp_min(0) if L["relu"] else x
            scales.append(_scale(x))
        elif kd == "dense":
            _, w, b = next(P)
            x = F.linear(x, tt(w), tt(b))
            x = x.clamp_min(0) if L["relu"] else x
            scales.append(_scale(x))
        elif kd == "maxpool":
            x = F.max_pool2d(x, L["k"], L["stride"], L["pad"])
        elif kd == "resblock":
            _, wa, ba = next(P)
            _, wb, bb = next(P)
            t = F.conv2d(x.clamp_min(0), tt(wa), tt(ba), padding=1).clamp_min(0)
            scales.append(_scale(t))
            x = x + F.conv2d(t, tt(wb), tt(bb), padding=1)
            scales.append(_scale(x))
        elif kd == "relu":
            x = x.clamp_min(0)
        elif kd == "flatten":
            x = x.flatten(1)
        elif kd == "lstm":
            break
    return np.asarray(scales, np.float32)


def quantize_policy(net, params, calib_states):
    """params: blob-order list of (name, W fp32, b fp32 or None).  Returns (tensors, act_scales) in the
    form pack_weights / pack_scales take."""
    has_lstm = any(L["kind"] == "lstm" for L in net.layers)
    tensors = []
    for name, w, b in params:
        if "lstm" in name or (name == "heads" and has_lstm):
            tensors.append(dict(name=name, w=np.asarray(w, np.float32), b=b))
        else:
            q, s = quantize_weight(w)
            tensors.append(dict(name=name, wq=q, s_w=s, b=np.asarray(b, np.float32)))
    return tensors, calibrate(net, params, calib_states)


def teacher_tensors(params):
    return [dict(name=n, w=np.asarray(w, np.float32), b=b) for n, w, b in params]


def _keep(l1, n_keep):
    order = np.lexsort((np.arange(l1.size), -l1))
    return np.sort(order[:n_keep])


def prune_policy(net_t, params_t, net_s):
    """Channel pruning by filter L1 norm down to the widths of net_s; convolutions writing one
    residual stream share their kept set (ranked by summed norm); hidden FC layers are kept whole."""
    P = {n: (np.asarray(w, np.float32), b) for n, w, b in params_t}
    l1 = lambda w: np.abs(w.astype(np.float64)).reshape(w.shape[0], -1).sum(axis=1)
    new, cur = {}, None
    shape = tuple(net_t.obs_shape)
    for i, (lt, ls) in enumerate(zip(net_t.layers, net_s.layers)):
        kd = lt["kind"]
        assert kd == ls["kind"]
        if kd == "conv":
            writers, j = [f"l{i}.conv"], i + 1
            while j < len(net_t.layers) and net_t.layers[j]["kind"] in ("maxpool", "resblock", "relu"):
                if net_t.layers[j]["kind"] == "resblock":
                    writers.append(f"l{j}.convB")
                j += 1
            keep = _keep(sum(l1(P[n][0]) for n in writers), ls["cout"])
            w, b = P[f"l{i}.conv"]
            w = w if cur is None else w[:, cur]
            new[f"l{i}.conv"] = (w[keep], b[keep])
            cur = keep
            h = (shape[1] + 2 * lt["pad"] - lt["k"]) // lt["stride"] + 1
            shape = (lt["cout"], h, h)
        elif kd == "maxpool":
            h = (shape[1] + 2 * lt["pad"] - lt["k"]) // lt["stride"] + 1
            shape = (shape[0], h, h)
        elif kd == "resblock":
            wa, ba = P[f"l{i}.convA"]
            wb, bb = P[f"l{i}.convB"]
            mid = _keep(l1(wa), ls["ch"])
            new[f"l{i}.convA"] = (wa[mid][:, cur], ba[mid])
            new[f"l{i}.convB"] = (wb[cur][:, mid], bb[cur])
        elif kd == "flatten":
            hw = shape[1] * shape[2]
            if cur is not None:
                cur = (cur[:, None] * hw + np.arange(hw)[None, :]).reshape(-1)
        elif kd == "dense":
            w, b = P[f"l{i}.dense"]
            new[f"l{i}.dense"] = (w if cur is None else w[:, cur], b)
            cur = None
        elif kd == "lstm":
            new[f"l{i}.lstm_ih"] = P[f"l{i}.lstm_ih"]
            new[f"l{i}.lstm_hh"] = P[f"l{i}.lstm_hh"]
    w, b = P["heads"]
    new["heads"] = (w if cur is None else w[:, cur], b)
    return [(n, np.ascontiguousarray(new[n][0]), None if new[n][1] is None else np.ascontiguousarray(new[n][1]))
            for n, _, _ in params_t]
