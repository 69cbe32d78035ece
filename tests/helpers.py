"""Shared test helpers: build teacher/student policies of a config with the oracle's PTQ."""
import functools

import numpy as np

import oracle
import workloads as wl


def make_states(net, B, stream, first=0):
    if net.obs_dtype == "u8":
        return wl.make_frames_u8(B, *net.obs_shape, stream=stream, first=first)
    return wl.make_obs_f32(B, net.obs_shape[0], stream=stream, first=first)


@functools.lru_cache(maxsize=None)
def policies(ci, calib=None):
    """(teacher net, teacher params, student net, student fp32 params, QuantPolicy)."""
    cfg = wl.CONFIGS[ci]
    nt, ns = cfg["teacher"], cfg["student"]
    pt = wl.init_params(nt, wl.STREAM["weights_teacher"])
    if cfg["student_from"] == "quantize":
        ps = pt
    elif cfg["student_from"] == "independent":
        ps = wl.init_params(ns, wl.STREAM["weights_student"])
    else:
        ps, _ = oracle.prune_policy(nt, pt, ns)
    n = calib or cfg["calib"]
    qp = oracle.quantize_policy(ns, ps, make_states(ns, n, wl.STREAM["calibration"]))
    return nt, pt, ns, ps, qp


def rel_err_rows(got, ref):
    """|got-ref| / max(|ref|, row max |ref|, 1e-6), per element; ref rows are states."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    if ref.ndim == 1:
        den = np.maximum(np.abs(ref).max(), 1e-6)
    else:
        den = np.maximum(np.abs(ref).max(axis=1, keepdims=True), 1e-6)
    return np.abs(got - ref) / den


# ------------------------------------------------------------------ GPU-side helpers
def student_tensors(qp):
    return qp.tensors


def teacher_tensors(params):
    return [dict(w=w, b=b) for _, w, b in params]


def action_margin(ref_logits, u):
    """Distance of each uniform to the nearest CDF boundary of the oracle's distribution (float64)."""
    l = np.asarray(ref_logits, np.float64)
    e = np.exp(l - l.max(axis=1, keepdims=True))
    cdf = np.cumsum(e, axis=1) / e.sum(axis=1, keepdims=True)
    return np.abs(cdf[:, :-1] - np.asarray(u, np.float64)[:, None]).min(axis=1) if l.shape[1] > 1 else np.ones(len(u))


def check_actions(got, ref_action, ref_logits, u, delta):
    got = np.asarray(got)
    assert got.min() >= 0 and got.max() < ref_logits.shape[1]
    bad = got != ref_action
    if bad.any():
        m = action_margin(ref_logits, u)
        assert np.all(m[bad] <= delta), f"{bad.sum()} actions differ, margins {m[bad][:8]}"
    return int(bad.sum())


def check_sampler_self_consistency(got_action, got_logits, u, delta=1e-5):
    """Sampler correctness apart from logit noise: the oracle's sampler run on the HIP path's OWN logits with the
    same uniforms must return the HIP path's actions, except where the uniform lies within delta of a boundary of
    that distribution's CDF (expf differs by ulps between the two sides)."""
    from oracle import layers as L
    got_logits = np.ascontiguousarray(got_logits, np.float32)
    u = np.ascontiguousarray(u, np.float32)
    want = L.softmax_sample(got_logits, u)
    return check_actions(got_action, want, got_logits, u, delta)
