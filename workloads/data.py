"""Recipes that turn the counter-based generator into the buffers of a workload.

Nothing here belongs to the method: uniform and normal draws, rectangles painted on
noise frames, uniform weight initialisation.  Every buffer is addressed by absolute
index, so `first` lets a caller regenerate rows first .. first+B-1 of a larger batch.
"""
import math

import numpy as np

from .rng import BASE_SEED, STREAM, u64, uniform01, normal, randint
from .nets import param_shapes

_CHUNK = 1 << 22  # words generated per numpy call, bounds temporary memory


def init_params(net, stream, seed=BASE_SEED):
    """Uniform init: W ~ U(+-sqrt(6/fan_in)), b ~ U(+-1/sqrt(fan_in)); fan_in = prod(W.shape[1:]).

    Returns a list of (name, W float32, b float32 or None) in blob order.  Each tensor
    draws from its own index range of the stream so shapes elsewhere do not shift it.
    """
    out = []
    for t, (name, wshape, bshape) in enumerate(param_shapes(net)):
        fan_in = int(np.prod(wshape[1:]))
        if "lstm" in name:
            fan_in = wshape[0] // 4          # hidden size, both matrices and the bias
            wb = 1.0 / math.sqrt(fan_in)
        else:
            wb = math.sqrt(6.0 / fan_in)
        bb = 1.0 / math.sqrt(fan_in)
        base = t << 32
        n = int(np.prod(wshape))
        w = (uniform01(seed, stream, base, n).astype(np.float64) * 2.0 - 1.0) * wb
        w = w.astype(np.float32).reshape(wshape)
        b = None
        if bshape is not None:
            nb = int(np.prod(bshape))
            b = ((uniform01(seed, stream, base + (1 << 31), nb).astype(np.float64) * 2.0 - 1.0) * bb).astype(np.float32)
        out.append((name, w, b))
    return out


def make_obs_f32(B, D, stream=STREAM["states"], first=0, seed=BASE_SEED):
    """float32 [B, D] ~ N(0, 1)."""
    return normal(seed, stream, first * D, B * D).reshape(B, D)


def make_uniforms(B, first=0, seed=BASE_SEED, stream=STREAM["uniforms"]):
    """float32 [B] in [0, 1)."""
    return uniform01(seed, stream, first, B)


def make_done(T, B, p=0.01, seed=BASE_SEED):
    """uint8 [T, B], Bernoulli(p)."""
    return (uniform01(seed, STREAM["done"], 0, T * B) < np.float32(p)).astype(np.uint8).reshape(T, B)


def make_hc(B, H, std=0.1, seed=BASE_SEED):
    """float32 h, c of shape [B, H] ~ N(0, std^2); c draws follow h's in the stream."""
    h = normal(seed, STREAM["hc"], 0, B * H).reshape(B, H) * np.float32(std)
    c = normal(seed, STREAM["hc"], B * H, B * H).reshape(B, H) * np.float32(std)
    return h.astype(np.float32), c.astype(np.float32)


def make_logits_pair(B, A, gap=0.3, scale=2.0, first=0, seed=BASE_SEED, stream=STREAM["monitor_logits"]):
    """Two float32 [B, A] logit tables standing for the original and the compressed policy on the same
    states: the first ~ scale * N(0, 1), the second = the first + gap * N(0, 1) (a compressed network
    tracks its teacher up to a perturbation)."""
    base = normal(seed, stream, 2 * first * A, B * A).reshape(B, A) * np.float32(scale)
    pert = normal(seed, stream + 100, 2 * first * A, B * A).reshape(B, A) * np.float32(gap)
    return base.astype(np.float32), (base + pert).astype(np.float32)


def make_trajectory(T, B, A, gamma=0.99, p_done=0.01, seed=BASE_SEED, stream=STREAM["trajectory"]):
    """One unroll of T steps for B environments, time-major: logits of both policies [T, B, A], the
    actions taken (uniform over A), rewards ~ N(0, 1) mostly zero (sparse, as in Atari), discounts
    gamma * (1 - done), values ~ N(0, 1) [T, B] and the bootstrap value [B]."""
    lo, ls = make_logits_pair(T * B, A, seed=seed, stream=stream)
    n = T * B
    actions = randint(seed, stream + 1, 0, n, 0, A - 1).astype(np.int32).reshape(T, B)
    rewards = (normal(seed, stream + 2, 0, n) * (uniform01(seed, stream + 3, 0, n) < np.float32(0.1))).astype(np.float32).reshape(T, B)
    done = uniform01(seed, stream + 4, 0, n) < np.float32(p_done)
    discounts = (np.float32(gamma) * (1.0 - done.astype(np.float32))).astype(np.float32).reshape(T, B)
    values = normal(seed, stream + 5, 0, n).reshape(T, B).astype(np.float32)
    bootstrap = normal(seed, stream + 6, 0, B).astype(np.float32)
    return dict(logits_original=lo.reshape(T, B, A), logits_smaller=ls.reshape(T, B, A), actions=actions,
                rewards=rewards, discounts=discounts, values=values, bootstrap=bootstrap)


def make_frames_u8(B, C=4, H=84, W=84, stream=STREAM["states"], first=0, n_rect=6, seed=BASE_SEED):
    """uint8 [B, C, H, W]: i.i.d. bytes, then per frame-channel n_rect constant rectangles.

    Rectangle r of plane p = (first+b)*C + c has width and height in 4..40, a position
    uniform among those that keep it inside the frame, and an intensity in 0..255; later
    rectangles overwrite earlier ones.  Stands in for Atari's flat regions.
    """
    plane = H * W
    out = np.empty((B, C, H, W), dtype=np.uint8)
    flat = out.reshape(-1)
    total = B * C * plane
    pos = 0
    while pos < total:
        n = min(_CHUNK, total - pos)
        flat[pos:pos + n] = (u64(seed, stream, first * C * plane + pos, n) >> np.uint64(56)).astype(np.uint8)
        pos += n
    # rectangle parameters: 5 words per rectangle
    rstream = STREAM["rectangles"] + 16 * stream
    ys = np.arange(H).reshape(1, 1, H, 1)
    xs = np.arange(W).reshape(1, 1, 1, W)
    step = 2048
    for b0 in range(0, B, step):
        nb = min(step, B - b0)
        npl = nb * C
        p0 = (first + b0) * C
        for r in range(n_rect):
            idx = (np.arange(p0, p0 + npl, dtype=np.int64) * n_rect + r) * 5
            rw = (_gather(seed, rstream, idx) % np.uint64(37)).astype(np.int64) + 4
            rh = (_gather(seed, rstream, idx + 1) % np.uint64(37)).astype(np.int64) + 4
            rw, rh = np.minimum(rw, W), np.minimum(rh, H)      # frames smaller than a rectangle: cut it to the frame
            x0 = (_gather(seed, rstream, idx + 2) % (W - rw + 1).astype(np.uint64)).astype(np.int64)
            y0 = (_gather(seed, rstream, idx + 3) % (H - rh + 1).astype(np.uint64)).astype(np.int64)
            val = (_gather(seed, rstream, idx + 4) >> np.uint64(56)).astype(np.uint8)
            shp = (nb, C, 1, 1)
            mask = ((ys >= y0.reshape(shp)) & (ys < (y0 + rh).reshape(shp)) &
                    (xs >= x0.reshape(shp)) & (xs < (x0 + rw).reshape(shp)))
            blk = out[b0:b0 + nb]
            np.copyto(blk, np.broadcast_to(val.reshape(shp), blk.shape), where=mask)
    return out


def _gather(seed, stream, idx):
    """64-bit words at arbitrary (int64 array) indices of a stream."""
    from .rng import _mix, _GOLD
    with np.errstate(over="ignore"):
        key = _mix(np.uint64(seed) * _GOLD + np.uint64(stream))
        return _mix(key + (idx.astype(np.uint64) + np.uint64(1)) * _GOLD)
