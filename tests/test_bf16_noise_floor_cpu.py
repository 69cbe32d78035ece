"""How far two correct bf16 implementations of the recurrent teacher may sit apart.

The oracle accumulates every dot product in fp64; hardware accumulates in fp32.  Both then round
each layer output to bfloat16, so a sum that lands near a rounding boundary flips by one bf16 ulp
(0.4-0.8 %) in one of them.  This test runs the same graph with library fp32 convolutions on the
CPU and measures the distance to the oracle: it stays below 2e-2 for the feed-forward IMPALA teacher
but not behind the LSTM, whose saturating gates amplify torso flips.  The GPU parity test of the
recurrent teacher takes its bounds (2e-2 at the 90th percentile, 6e-2 worst case) from here.
"""
import numpy as np
import torch
import torch.nn.functional as F

import oracle
import workloads as wl
from helpers import policies, make_states, rel_err_rows


def bf(t):
    return t.to(torch.bfloat16).to(torch.float32)


@torch.no_grad()
def fp32_accumulating_teacher(net, params, x8, h=None, c=None, done=None):
    P = iter(params)
    tt = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    x = bf(torch.from_numpy(x8).float() / 255.0)
    for ly in net.layers:
        kd = ly["kind"]
        if kd == "conv":
            _, w, b = next(P)
            x = F.conv2d(x, bf(tt(w)), None, stride=ly["stride"], padding=ly["pad"]) + tt(b).view(1, -1, 1, 1)
            x = bf(x.clamp_min(0) if ly["relu"] else x)
        elif kd == "maxpool":
            x = F.max_pool2d(x, ly["k"], ly["stride"], ly["pad"])
        elif kd == "resblock":
            _, wa, ba = next(P)
            _, wb, bb = next(P)
            t = bf((F.conv2d(x.clamp_min(0), bf(tt(wa)), None, padding=1) + tt(ba).view(1, -1, 1, 1)).clamp_min(0))
            x = bf(x + (F.conv2d(t, bf(tt(wb)), None, padding=1) + tt(bb).view(1, -1, 1, 1)))
        elif kd == "relu":
            x = x.clamp_min(0)
        elif kd == "flatten":
            x = x.flatten(1)
        elif kd == "dense":
            _, w, b = next(P)
            x = bf((F.linear(x, bf(tt(w))) + tt(b)).clamp_min(0))
        elif kd == "lstm":
            _, wih, bi = next(P)
            _, whh, _ = next(P)
            h, c = torch.from_numpy(h.copy()), torch.from_numpy(c.copy())
            m = torch.from_numpy(done.astype(bool))
            h[m] = 0
            c[m] = 0
            g = F.linear(x, bf(tt(wih))) + F.linear(bf(h), bf(tt(whh))) + tt(bi)
            i, f, gg, o = g.chunk(4, 1)
            c = torch.sigmoid(f) * c + torch.sigmoid(i) * torch.tanh(gg)
            x = torch.sigmoid(o) * torch.tanh(c)
    _, wh, bh = next(P)
    return (F.linear(bf(x), bf(tt(wh))) + tt(bh)).numpy()


def test_bf16_noise_floor():
    B = 48
    res = {}
    for ci in (3, 4):
        nt, pt, _, _, _ = policies(ci, 16)
        x = make_states(nt, B, wl.STREAM["states"])
        kw = {}
        if ci == 4:
            h0, c0 = wl.make_hc(B, 256)
            kw = dict(h=h0, c=c0, done=wl.make_done(1, B, p=0.2)[0])
        ref = oracle.forward_float(nt, pt, x, None, "bf16", **kw)
        out = fp32_accumulating_teacher(nt, pt, x, **kw)
        res[ci] = rel_err_rows(out[:, :18], ref["logits"])
    assert res[3].max() < 2e-2                      # feed-forward teacher: inside the stated bar
    assert np.quantile(res[4], 0.9) < 2e-2          # recurrent teacher: bulk inside ...
    assert 5e-3 < res[4].max() < 6e-2               # ... the worst element is not, on either side
