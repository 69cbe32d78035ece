"""Layer lists of the policy networks (shapes only, no arithmetic).

A Net is an observation description, a list of layers and a number of actions; two
heads (A logits, 1 value) always follow the last layer.  Layers are plain dicts:

  conv     cin cout k stride pad relu     (square kernel, symmetric zero padding)
  dense    cin cout relu
  maxpool  k stride pad                   (padding taps are ignored)
  resblock ch                             (x + convB(relu(convA(relu(x)))), 3x3 pad 1)
  relu
  flatten                                 (C,H,W order)
  lstm     cin hidden                     (gate order i, f, g, o)
"""
from dataclasses import dataclass, field
from typing import List, Tuple


def conv(cin, cout, k, stride=1, pad=0, relu=True):
    return dict(kind="conv", cin=cin, cout=cout, k=k, stride=stride, pad=pad, relu=bool(relu))


def dense(cin, cout, relu=True):
    return dict(kind="dense", cin=cin, cout=cout, relu=bool(relu))


def maxpool(k=3, stride=2, pad=1):
    return dict(kind="maxpool", k=k, stride=stride, pad=pad)


def resblock(ch):
    return dict(kind="resblock", ch=ch)


def relu():
    return dict(kind="relu")


def flatten():
    return dict(kind="flatten")


def lstm(cin, hidden):
    return dict(kind="lstm", cin=cin, hidden=hidden)


@dataclass
class Net:
    name: str
    obs_dtype: str                 # "u8" or "f32"
    obs_shape: Tuple[int, ...]     # (D,) or (C, H, W)
    n_actions: int
    layers: List[dict] = field(default_factory=list)


def _out_hw(h, k, s, p):
    return (h + 2 * p - k) // s + 1


def trace_shapes(net):
    """Shape of the tensor after each layer: list of tuples, (C,H,W) or (D,)."""
    shp = tuple(net.obs_shape)
    out = []
    for L in net.layers:
        kd = L["kind"]
        if kd == "conv":
            c, h, w = shp
            assert c == L["cin"], (net.name, L, shp)
            shp = (L["cout"], _out_hw(h, L["k"], L["stride"], L["pad"]), _out_hw(w, L["k"], L["stride"], L["pad"]))
        elif kd == "maxpool":
            c, h, w = shp
            shp = (c, _out_hw(h, L["k"], L["stride"], L["pad"]), _out_hw(w, L["k"], L["stride"], L["pad"]))
        elif kd == "resblock":
            assert shp[0] == L["ch"], (net.name, L, shp)
        elif kd == "relu":
            pass
        elif kd == "flatten":
            n = 1
            for d in shp:
                n *= d
            shp = (n,)
        elif kd == "dense":
            assert shp == (L["cin"],), (net.name, L, shp)
            shp = (L["cout"],)
        elif kd == "lstm":
            assert shp == (L["cin"],), (net.name, L, shp)
            shp = (L["hidden"],)
        else:
            raise ValueError(kd)
        out.append(shp)
    return out


def feature_dim(net):
    shp = trace_shapes(net)[-1] if net.layers else tuple(net.obs_shape)
    assert len(shp) == 1, "heads need a flat feature vector"
    return shp[0]


def param_shapes(net):
    """(name, weight shape, bias shape) of every parametrised tensor pair, in blob order."""
    out = []
    for i, L in enumerate(net.layers):
        kd = L["kind"]
        if kd == "conv":
            out.append((f"l{i}.conv", (L["cout"], L["cin"], L["k"], L["k"]), (L["cout"],)))
        elif kd == "dense":
            out.append((f"l{i}.dense", (L["cout"], L["cin"]), (L["cout"],)))
        elif kd == "resblock":
            out.append((f"l{i}.convA", (L["ch"], L["ch"], 3, 3), (L["ch"],)))
            out.append((f"l{i}.convB", (L["ch"], L["ch"], 3, 3), (L["ch"],)))
        elif kd == "lstm":
            out.append((f"l{i}.lstm_ih", (4 * L["hidden"], L["cin"]), (4 * L["hidden"],)))
            out.append((f"l{i}.lstm_hh", (4 * L["hidden"], L["hidden"]), None))
    out.append(("heads", (net.n_actions + 1, feature_dim(net)), (net.n_actions + 1,)))
    return out


def mlp(name, d_in, hidden, n_actions):
    layers, c = [], d_in
    for h in hidden:
        layers.append(dense(c, h, True))
        c = h
    return Net(name, "f32", (d_in,), n_actions, layers)


def nature_cnn(name="nature_cnn", n_actions=18, fc=512):
    return Net(name, "u8", (4, 84, 84), n_actions, [
        conv(4, 32, 8, 4, 0, True), conv(32, 64, 4, 2, 0, True), conv(64, 64, 3, 1, 0, True),
        flatten(), dense(64 * 7 * 7, fc, True)])


def paper_small_cnn(name, c1, c2, fc, n_actions=18):
    """The two-conv students of the paper's network table (filters 8 and 4, strides 4 and 2)."""
    return Net(name, "u8", (4, 84, 84), n_actions, [
        conv(4, c1, 8, 4, 0, True), conv(c1, c2, 4, 2, 0, True),
        flatten(), dense(c2 * 9 * 9, fc, True)])


def impala_cnn(name, channels=(16, 32, 32), n_actions=18, fc=256, lstm_hidden=0):
    layers, c, hw = [], 4, 84
    for ch in channels:
        layers += [conv(c, ch, 3, 1, 1, False), maxpool(3, 2, 1), resblock(ch), resblock(ch)]
        c, hw = ch, _out_hw(hw, 3, 2, 1)
    layers += [relu(), flatten(), dense(c * hw * hw, fc, True)]
    if lstm_hidden:
        layers.append(lstm(fc, lstm_hidden))
    return Net(name, "u8", (4, 84, 84), n_actions, layers)
