"""ctypes binding of include/accerl.h: same names, argument marshalling only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libaccerl.so")
_lib = None

INT8, FP32, BF16 = 0, 1, 2
OBS_U8, OBS_F32 = 0, 1
TAP_ACC, TAP_ACT, TAP_ACC_A, TAP_ACT_A = 0, 1, 2, 3
MAX_LAYERS = 48
_KINDS = {"conv": 1, "dense": 2, "maxpool": 3, "resblock": 4, "relu": 5, "flatten": 6, "lstm": 7}
_PREC = {"int8": INT8, "fp32": FP32, "bf16": BF16}


class AccerlError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"accerl status {code}: {msg}")
        self.code = code


class _Layer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "cin", "cout", "k", "stride", "pad", "relu", "reserved")]


class _Arch(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("obs_dtype", "obs_c", "obs_h", "obs_w", "n_actions", "precision", "n_layers")] + \
               [("layers", _Layer * MAX_LAYERS)]


def load_library():
    """Load libaccerl.so (after torch, so that both share one HIP runtime).  No fallback exists."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  -- brings in the HIP runtime the library links against
    if not os.path.exists(_SO):
        raise ImportError(f"{_SO} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or paper_2211_15023_amd/build.py); there is no CPU fallback")
    lib = C.CDLL(_SO)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    lib.accerl_blob_sizes.argtypes = [C.POINTER(_Arch), C.POINTER(i64), C.POINTER(i64)]
    lib.accerl_policy_create.argtypes = [C.POINTER(_Arch), vp, i64, vp, i64, C.POINTER(vp)]
    lib.accerl_policy_destroy.argtypes = [vp]
    lib.accerl_policy_destroy.restype = None
    fwd = [vp, vp, i64, vp, vp, vp, vp, vp]
    lib.accerl_actor_forward.argtypes = fwd
    lib.accerl_actor_forward_teacher.argtypes = fwd
    lib.accerl_actor_forward_recurrent.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.accerl_actor_forward_debug.argtypes = [vp, vp, i64, i32, i32, vp, i64, vp]
    lib.accerl_plan_describe.argtypes = [C.POINTER(_Arch), vp, i64, vp, i64, C.c_char_p, i64]
    lib.accerl_plan_describe.restype = C.c_int
    lib.accerl_profile_begin.argtypes = [vp]
    lib.accerl_profile_end.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.accerl_monitor_kl.argtypes = [vp, vp, i64, i32, vp, vp, vp, vp]
    lib.accerl_vtrace.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i32, C.c_float, C.c_float, vp, vp, vp, vp]
    lib.accerl_monitor_kl.restype = C.c_int
    lib.accerl_monitor_kl_noalloc.argtypes = [vp, vp, i64, i32, vp, vp, vp, vp]
    lib.accerl_monitor_kl_noalloc.restype = C.c_int
    lib.accerl_probe_mfma.argtypes = [i32, i32, vp, vp]
    lib.accerl_probe_mfma.restype = C.c_int
    lib.accerl_probe_copy.argtypes = [vp, vp, i64, vp]
    lib.accerl_probe_copy.restype = C.c_int
    lib.accerl_probe_empty.argtypes = [vp]
    lib.accerl_probe_empty.restype = C.c_int
    lib.accerl_actor_forward_mixture.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.accerl_actor_forward_mixture.restype = C.c_int
    lib.accerl_mixture_alpha.argtypes = [C.c_double, C.c_double, C.c_double]
    lib.accerl_mixture_alpha.restype = C.c_double
    lib.accerl_distill_loss.argtypes = [vp, vp, vp, vp, i64, i32, C.c_float, vp, vp, vp]
    lib.accerl_distill_loss.restype = C.c_int
    lib.accerl_vtrace.restype = C.c_int
    lib.accerl_last_error.restype = C.c_char_p
    for f in ("accerl_blob_sizes", "accerl_policy_create", "accerl_actor_forward", "accerl_actor_forward_teacher",
              "accerl_actor_forward_recurrent", "accerl_actor_forward_debug", "accerl_profile_begin",
              "accerl_profile_end"):
        getattr(lib, f).restype = C.c_int
    _lib = lib
    return lib


def accerl_last_error():
    return load_library().accerl_last_error().decode()


def _check(rc):
    if rc != 0:
        raise AccerlError(rc, accerl_last_error())


def make_arch(net, precision):
    """net: object with obs_dtype ("u8"/"f32"), obs_shape, n_actions, layers (list of dicts)."""
    a = _Arch()
    a.obs_dtype = OBS_U8 if net.obs_dtype == "u8" else OBS_F32
    shp = tuple(net.obs_shape)
    a.obs_c, a.obs_h, a.obs_w = (shp[0], 1, 1) if len(shp) == 1 else shp
    a.n_actions = net.n_actions
    a.precision = _PREC[precision] if isinstance(precision, str) else int(precision)
    if len(net.layers) > MAX_LAYERS:
        raise ValueError("too many layers")
    a.n_layers = len(net.layers)
    for i, L in enumerate(net.layers):
        l = a.layers[i]
        l.kind = _KINDS[L["kind"]]
        if L["kind"] == "resblock":
            l.cin = l.cout = L["ch"]
        elif L["kind"] == "lstm":
            l.cin, l.cout = L["cin"], L["hidden"]
        else:
            l.cin, l.cout = L.get("cin", 0), L.get("cout", 0)
        l.k, l.stride, l.pad = L.get("k", 0), L.get("stride", 0), L.get("pad", 0)
        l.relu = int(bool(L.get("relu", False)))
    return a


def blob_sizes(arch):
    wb, ns = C.c_int64(), C.c_int64()
    _check(load_library().accerl_blob_sizes(C.byref(arch), C.byref(wb), C.byref(ns)))
    return wb.value, ns.value


def pack_weights(tensors):
    """tensors: blob-order list of dicts with "wq" (int8) or "w" (fp32) and "b" (fp32 or None).
    For an LSTM the pair is (W_ih with the bias, W_hh without).  Returns a uint8 array."""
    out = bytearray()

    def put(arr):
        pad = (-len(out)) % 16
        out.extend(b"\0" * pad)
        out.extend(np.ascontiguousarray(arr).tobytes())

    for t in tensors:
        if "wq" in t:
            put(np.asarray(t["wq"], np.int8))
        else:
            put(np.asarray(t["w"], np.float32))
        if t.get("b") is not None:
            put(np.asarray(t["b"], np.float32))
    return np.frombuffer(bytes(out), np.uint8)


def pack_scales(act_scales, tensors):
    parts = [np.asarray(act_scales, np.float32).reshape(-1)]
    parts += [np.asarray(t["s_w"], np.float32).reshape(-1) for t in tensors if "wq" in t]
    return np.ascontiguousarray(np.concatenate(parts))


def accerl_policy_create(arch, weights, quant_scales=None):
    """weights: uint8 numpy blob; quant_scales: float32 numpy array or None.  Returns an opaque handle."""
    lib = load_library()
    weights = np.ascontiguousarray(weights, np.uint8)
    ns, sp = 0, None
    if quant_scales is not None and len(quant_scales):
        quant_scales = np.ascontiguousarray(quant_scales, np.float32)
        ns, sp = quant_scales.size, quant_scales.ctypes.data_as(C.c_void_p)
    h = C.c_void_p()
    _check(lib.accerl_policy_create(C.byref(arch), weights.ctypes.data_as(C.c_void_p), weights.size, sp, ns, C.byref(h)))
    return h


def accerl_plan_describe(arch, weights, quant_scales=None):
    """Text description of the launch plan (host only, no GPU needed)."""
    lib = load_library()
    weights = np.ascontiguousarray(weights, np.uint8)
    ns, sp = 0, None
    if quant_scales is not None and len(quant_scales):
        quant_scales = np.ascontiguousarray(quant_scales, np.float32)
        ns, sp = quant_scales.size, quant_scales.ctypes.data_as(C.c_void_p)
    buf = C.create_string_buffer(1 << 16)
    _check(lib.accerl_plan_describe(C.byref(arch), weights.ctypes.data_as(C.c_void_p), weights.size, sp, ns, buf, len(buf)))
    return buf.value.decode()


def accerl_policy_destroy(handle):
    load_library().accerl_policy_destroy(handle)


def _ptr(t, dtype=None):
    import torch
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device tensors must be contiguous CUDA/HIP tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def accerl_actor_forward(handle, states, uniforms, out_logits, out_value, out_action, stream=None):
    import torch
    B = states.shape[0]
    _check(load_library().accerl_actor_forward(handle, _ptr(states), B, _ptr(uniforms, torch.float32),
                                               _ptr(out_logits, torch.float32), _ptr(out_value, torch.float32),
                                               _ptr(out_action, torch.int32), _stream(stream)))


def accerl_actor_forward_teacher(handle, states, uniforms, out_logits, out_value, out_action, stream=None):
    import torch
    B = states.shape[0]
    _check(load_library().accerl_actor_forward_teacher(handle, _ptr(states), B, _ptr(uniforms, torch.float32),
                                                       _ptr(out_logits, torch.float32), _ptr(out_value, torch.float32),
                                                       _ptr(out_action, torch.int32), _stream(stream)))


def accerl_actor_forward_recurrent(handle, states, uniforms, done, h, c, out_logits, out_value, out_action, stream=None):
    import torch
    B = states.shape[0]
    _check(load_library().accerl_actor_forward_recurrent(
        handle, _ptr(states), B, _ptr(uniforms, torch.float32), _ptr(done, torch.uint8), _ptr(h, torch.float32),
        _ptr(c, torch.float32), _ptr(out_logits, torch.float32), _ptr(out_value, torch.float32),
        _ptr(out_action, torch.int32), _stream(stream)))


def accerl_actor_forward_debug(handle, states, layer, tap, out, stream=None):
    B = states.shape[0]
    _check(load_library().accerl_actor_forward_debug(handle, _ptr(states), B, int(layer), int(tap), _ptr(out),
                                                     out.numel() * out.element_size(), _stream(stream)))


def accerl_actor_forward_mixture(smaller, original, states, uniforms, use_smaller, out_logits, out_value, out_action, stream=None):
    """use_smaller: host uint8 array [B] (numpy); the other tensors live on the device."""
    import numpy as np
    import torch
    B = states.shape[0]
    flags = np.ascontiguousarray(use_smaller, dtype=np.uint8)
    if flags.shape != (B,):
        raise ValueError("use_smaller must be a host array of B flags")
    _check(load_library().accerl_actor_forward_mixture(smaller, original, _ptr(states), B, _ptr(uniforms, torch.float32),
                                                       flags.ctypes.data_as(C.c_void_p), _ptr(out_logits, torch.float32),
                                                       _ptr(out_value, torch.float32), _ptr(out_action, torch.int32),
                                                       _stream(stream)))


def accerl_mixture_alpha(kl_mean, kl_lo, kl_hi):
    return float(load_library().accerl_mixture_alpha(kl_mean, kl_lo, kl_hi))


def accerl_probe_mfma(bf16, iters, sink, stream=None):
    import torch
    _check(load_library().accerl_probe_mfma(int(bool(bf16)), int(iters), _ptr(sink, torch.int32), _stream(stream)))


def accerl_probe_copy(src, dst, stream=None):
    n = src.numel() * src.element_size()
    _check(load_library().accerl_probe_copy(_ptr(src), _ptr(dst), n, _stream(stream)))


def accerl_probe_empty(stream=None):
    _check(load_library().accerl_probe_empty(_stream(stream)))


def accerl_monitor_kl(logits_original, logits_smaller, out_kl, out_entropy, out_stats, stream=None):
    """out_stats: float64 device tensor [4] = KL mean, KL max, KL variance, entropy mean."""
    import torch
    B, A = logits_original.shape
    if tuple(logits_smaller.shape) != (B, A):
        raise ValueError("logit tables differ in shape")
    _check(load_library().accerl_monitor_kl(_ptr(logits_original, torch.float32), _ptr(logits_smaller, torch.float32), B, A,
                                            _ptr(out_kl, torch.float32), _ptr(out_entropy, torch.float32),
                                            _ptr(out_stats, torch.float64), _stream(stream)))


def accerl_monitor_kl_noalloc(logits_original, logits_smaller, out_kl, out_entropy, out_stats, stream=None):
    """accerl_monitor_kl on the library's fixed partial-sum array: no device allocation, at most 2^24 rows."""
    import torch
    B, A = logits_original.shape
    if tuple(logits_smaller.shape) != (B, A):
        raise ValueError("logit tables differ in shape")
    _check(load_library().accerl_monitor_kl_noalloc(_ptr(logits_original, torch.float32), _ptr(logits_smaller, torch.float32), B, A,
                                                    _ptr(out_kl, torch.float32), _ptr(out_entropy, torch.float32),
                                                    _ptr(out_stats, torch.float64), _stream(stream)))


def accerl_distill_loss(logits_original, logits_smaller, value_original, value_smaller, beta, out_loss, out_mean, stream=None):
    import torch
    B, A = logits_original.shape
    if tuple(logits_smaller.shape) != (B, A) or tuple(value_original.shape) != (B,) or tuple(value_smaller.shape) != (B,):
        raise ValueError("shapes differ")
    _check(load_library().accerl_distill_loss(_ptr(logits_original, torch.float32), _ptr(logits_smaller, torch.float32),
                                              _ptr(value_original, torch.float32), _ptr(value_smaller, torch.float32), B, A,
                                              float(beta), _ptr(out_loss, torch.float32), _ptr(out_mean, torch.float64),
                                              _stream(stream)))


def accerl_vtrace(logits_original, logits_smaller, actions, rewards, discounts, values, bootstrap,
                  rho_bar, c_bar, out_vs, out_pg_adv, out_rho, stream=None):
    import torch
    T, B, A = logits_original.shape
    if tuple(logits_smaller.shape) != (T, B, A):
        raise ValueError("logit tables differ in shape")
    for t in (actions, rewards, discounts, values, out_vs, out_rho):
        if tuple(t.shape) != (T, B):
            raise ValueError("per-step tensors must be [T, B]")
    _check(load_library().accerl_vtrace(_ptr(logits_original, torch.float32), _ptr(logits_smaller, torch.float32),
                                        _ptr(actions, torch.int32), _ptr(rewards, torch.float32), _ptr(discounts, torch.float32),
                                        _ptr(values, torch.float32), _ptr(bootstrap, torch.float32), T, B, A,
                                        float(rho_bar), float(c_bar), _ptr(out_vs, torch.float32),
                                        _ptr(out_pg_adv, torch.float32), _ptr(out_rho, torch.float32), _stream(stream)))


STEP_KINDS = ("mlp_fused", "quant_obs", "conv", "gemm", "gemm_f32", "maxpool", "lstm_pack", "sample", "heads")


def accerl_profile_begin(handle):
    _check(load_library().accerl_profile_begin(handle))


def accerl_profile_end(handle):
    """Returns a list of dicts: step, layer, kind, launches, total_ms."""
    cap = 256
    n = C.c_int32()
    ms = (C.c_float * cap)()
    cnt = (C.c_int64 * cap)()
    layer = (C.c_int32 * cap)()
    kind = (C.c_int32 * cap)()
    _check(load_library().accerl_profile_end(handle, cap, C.byref(n), ms, cnt, layer, kind))
    return [dict(step=i, layer=layer[i], kind=STEP_KINDS[kind[i]], launches=cnt[i], total_ms=ms[i])
            for i in range(n.value)]


class Policy:
    """Convenience owner of a policy handle plus output allocation through torch."""

    def __init__(self, net, precision, tensors, act_scales=None):
        self.net = net
        self.precision = precision
        self.arch = make_arch(net, precision)
        blob = pack_weights(tensors)
        scales = pack_scales(act_scales, tensors) if precision == "int8" else None
        self.handle = accerl_policy_create(self.arch, blob, scales)
        self.recurrent = any(L["kind"] == "lstm" for L in net.layers)

    def close(self):
        if self.handle is not None:
            accerl_policy_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def alloc_outputs(self, B, device="cuda"):
        import torch
        A = self.net.n_actions
        return (torch.empty((B, A), dtype=torch.float32, device=device),
                torch.empty((B,), dtype=torch.float32, device=device),
                torch.empty((B,), dtype=torch.int32, device=device))

    def forward(self, states, uniforms, done=None, h=None, c=None, outputs=None, stream=None):
        logits, value, action = outputs if outputs is not None else self.alloc_outputs(states.shape[0], states.device)
        if self.recurrent:
            accerl_actor_forward_recurrent(self.handle, states, uniforms, done, h, c, logits, value, action, stream)
        elif self.precision == "int8":
            accerl_actor_forward(self.handle, states, uniforms, logits, value, action, stream)
        else:
            accerl_actor_forward_teacher(self.handle, states, uniforms, logits, value, action, stream)
        return logits, value, action

    def tap(self, states, layer, tap, shape, dtype, stream=None):
        import torch
        out = torch.empty(shape, dtype=dtype, device=states.device)
        accerl_actor_forward_debug(self.handle, states, layer, tap, out, stream)
        return out
