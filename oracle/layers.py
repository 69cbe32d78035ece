"""numpy-facing wrappers of the C layer functions (argument marshalling only)."""
import ctypes as C

import numpy as np

from .clib import lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def _ohw(h, k, s, p):
    return (h + 2 * p - k) // s + 1


def num_threads():
    return lib().orc_num_threads()


def set_threads(n):
    lib().orc_set_threads(C.c_int(n))


def bf16_round(x):
    x = _c(x, np.float32)
    y = np.empty_like(x)
    lib().orc_bf16_round(_p(x), C.c_int64(x.size), _p(y))
    return y


def conv2d_f(x, w, b, stride, pad, relu, bf16):
    x, w, b = _c(x, np.float32), _c(w, np.float32), _c(b, np.float32)
    B, Ci, H, W = x.shape
    Co, Ci2, k, k2 = w.shape
    assert Ci == Ci2 and k == k2 and b.shape == (Co,)
    y = np.empty((B, Co, _ohw(H, k, stride, pad), _ohw(W, k, stride, pad)), np.float32)
    lib().orc_conv2d_f(_p(x), C.c_int64(B), Ci, H, W, _p(w), _p(b), Co, k, stride, pad,
                       int(relu), int(bf16), _p(y))
    return y


def dense_f(x, w, b, relu, bf16):
    x, w = _c(x, np.float32), _c(w, np.float32)
    B, K = x.shape
    N, K2 = w.shape
    assert K == K2
    if b is not None:
        b = _c(b, np.float32)
        assert b.shape == (N,)
    y = np.empty((B, N), np.float32)
    lib().orc_dense_f(_p(x), C.c_int64(B), K, _p(w), _p(b) if b is not None else None, N,
                      int(relu), int(bf16), _p(y))
    return y


def maxpool_f(x, k, s, p):
    x = _c(x, np.float32)
    B, Ci, H, W = x.shape
    y = np.empty((B, Ci, _ohw(H, k, s, p), _ohw(W, k, s, p)), np.float32)
    lib().orc_maxpool_f(_p(x), C.c_int64(B), Ci, H, W, k, s, p, _p(y))
    return y


def quantize_f32(x, inv_s):
    x = _c(x, np.float32)
    q = np.empty(x.shape, np.int8)
    lib().orc_quantize_f32(_p(x), C.c_int64(x.size), C.c_float(inv_s), _p(q))
    return q


def conv2d_q_acc(x, wq, biasq, stride, pad, relu_in=False):
    assert x.dtype in (np.uint8, np.int8)
    x = np.ascontiguousarray(x)
    wq, biasq = _c(wq, np.int8), _c(biasq, np.int32)
    B, Ci, H, W = x.shape
    Co, Ci2, k, k2 = wq.shape
    assert Ci == Ci2 and k == k2 and biasq.shape == (Co,)
    acc = np.empty((B, Co, _ohw(H, k, stride, pad), _ohw(W, k, stride, pad)), np.int32)
    lib().orc_conv2d_q_acc(_p(x), int(x.dtype == np.uint8), int(relu_in), C.c_int64(B), Ci, H, W,
                           _p(wq), _p(biasq), Co, k, stride, pad, _p(acc))
    return acc


def dense_q_acc(x, wq, biasq, relu_in=False):
    x, wq, biasq = _c(x, np.int8), _c(wq, np.int8), _c(biasq, np.int32)
    B, K = x.shape
    N, K2 = wq.shape
    assert K == K2 and biasq.shape == (N,)
    acc = np.empty((B, N), np.int32)
    lib().orc_dense_q_acc(_p(x), int(relu_in), C.c_int64(B), K, _p(wq), _p(biasq), N, _p(acc))
    return acc


def requant(acc, m, lo):
    acc, m = _c(acc, np.int32), _c(m, np.float32)
    B, Cn = acc.shape[:2]
    hw = int(np.prod(acc.shape[2:])) if acc.ndim > 2 else 1
    assert m.shape == (Cn,)
    q = np.empty(acc.shape, np.int8)
    lib().orc_requant(_p(acc), C.c_int64(B), Cn, hw, _p(m), int(lo), _p(q))
    return q


def requant_residual(acc, xq, r, m):
    acc, xq, m = _c(acc, np.int32), _c(xq, np.int8), _c(m, np.float32)
    assert acc.shape == xq.shape
    B, Cn = acc.shape[:2]
    hw = int(np.prod(acc.shape[2:])) if acc.ndim > 2 else 1
    q = np.empty(acc.shape, np.int8)
    lib().orc_requant_residual(_p(acc), _p(xq), C.c_float(r), C.c_int64(B), Cn, hw, _p(m), _p(q))
    return q


def maxpool_i8(x, k, s, p):
    x = _c(x, np.int8)
    B, Ci, H, W = x.shape
    y = np.empty((B, Ci, _ohw(H, k, s, p), _ohw(W, k, s, p)), np.int8)
    lib().orc_maxpool_i8(_p(x), C.c_int64(B), Ci, H, W, k, s, p, _p(y))
    return y


def dequant(acc, d):
    acc, d = _c(acc, np.int32), _c(d, np.float32)
    B, N = acc.shape
    out = np.empty((B, N), np.float32)
    lib().orc_dequant(_p(acc), C.c_int64(B), N, _p(d), _p(out))
    return out


def dequant_i8(q, s):
    q = _c(q, np.int8)
    x = np.empty(q.shape, np.float32)
    lib().orc_dequant_i8(_p(q), C.c_int64(q.size), C.c_float(s), _p(x))
    return x


def softmax_sample(logits, u, want_logp=False):
    logits, u = _c(logits, np.float32), _c(u, np.float32)
    B, A = logits.shape
    assert u.shape == (B,)
    act = np.empty(B, np.int32)
    logp = np.empty((B, A), np.float32) if want_logp else None
    lib().orc_softmax_sample(_p(logits), C.c_int64(B), A, _p(u), _p(act),
                             _p(logp) if want_logp else None)
    return (act, logp) if want_logp else act


def lstm_step(x, h, c, done, w_ih, w_hh, bias, bf16):
    """Returns new (h, c); inputs are not modified."""
    x, w_ih, w_hh, bias = _c(x, np.float32), _c(w_ih, np.float32), _c(w_hh, np.float32), _c(bias, np.float32)
    h = np.array(h, dtype=np.float32, order="C", copy=True)
    c = np.array(c, dtype=np.float32, order="C", copy=True)
    B, In = x.shape
    Hd = h.shape[1]
    assert h.shape == c.shape == (B, Hd) and w_ih.shape == (4 * Hd, In) and w_hh.shape == (4 * Hd, Hd)
    assert Hd <= 1024 and bias.shape == (4 * Hd,)
    if done is not None:
        done = _c(done, np.uint8)
        assert done.shape == (B,)
    lib().orc_lstm_step(_p(x), C.c_int64(B), In, Hd, _p(done) if done is not None else None,
                        _p(w_ih), _p(w_hh), _p(bias), int(bf16), _p(h), _p(c))
    return h, c


def kl_monitor(logits_original, logits_smaller):
    """Monitor indicators: per-state KL(original || smaller), entropy of the smaller policy,
    stats = [KL mean, KL max, KL variance, entropy mean] (all float64)."""
    lo, ls = _c(logits_original, np.float32), _c(logits_smaller, np.float32)
    B, A = lo.shape
    assert ls.shape == (B, A) and A <= 256
    kl = np.empty(B, np.float64)
    ent = np.empty(B, np.float64)
    stats = np.empty(4, np.float64)
    lib().orc_kl_monitor(_p(lo), _p(ls), C.c_int64(B), A, _p(kl), _p(ent), _p(stats))
    return kl, ent, stats


def vtrace(logits_original, logits_smaller, actions, rewards, discounts, values, bootstrap,
           rho_bar=1.0, c_bar=1.0):
    """V-trace targets v_s, importance-weighted advantages and rho_t, time-major [T, B]."""
    lo, ls = _c(logits_original, np.float32), _c(logits_smaller, np.float32)
    T, B, A = lo.shape
    assert ls.shape == (T, B, A) and A <= 256 and T <= 4096
    a = _c(actions, np.int32)
    r, d, v = _c(rewards, np.float32), _c(discounts, np.float32), _c(values, np.float32)
    bs = _c(bootstrap, np.float32)
    assert a.shape == r.shape == d.shape == v.shape == (T, B) and bs.shape == (B,)
    assert a.min() >= 0 and a.max() < A
    vs = np.empty((T, B), np.float64)
    adv = np.empty((T, B), np.float64)
    rho = np.empty((T, B), np.float64)
    lib().orc_vtrace(_p(lo), _p(ls), _p(a), _p(r), _p(d), _p(v), _p(bs), C.c_int64(T), C.c_int64(B), A,
                     C.c_double(rho_bar), C.c_double(c_bar), _p(vs), _p(adv), _p(rho))
    return vs, adv, rho


def distill_loss(logits_original, logits_smaller, v_original, v_smaller, beta):
    """Knowledge-distillation loss per state and its batch mean (float64)."""
    lo, ls = _c(logits_original, np.float32), _c(logits_smaller, np.float32)
    vo, vs = _c(v_original, np.float32), _c(v_smaller, np.float32)
    B, A = lo.shape
    assert ls.shape == (B, A) and vo.shape == (B,) and vs.shape == (B,) and A <= 256
    loss = np.empty(B, np.float64)
    mean = np.empty(1, np.float64)
    lib().orc_distill_loss(_p(lo), _p(ls), _p(vo), _p(vs), C.c_int64(B), A, C.c_double(beta), _p(loss), _p(mean))
    return loss, float(mean[0])


def mixture_alpha(kl_mean, kl_lo, kl_hi):
    f = lib().orc_mixture_alpha
    f.restype = C.c_double
    return float(f(C.c_double(kl_mean), C.c_double(kl_lo), C.c_double(kl_hi)))
