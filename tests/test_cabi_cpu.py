"""The C-ABI library loads, exports every declared symbol and rejects bad arguments without a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def A():
    import paper_2211_15023_amd as A
    A.load_library()
    return A


def test_exports_every_declared_symbol(A):
    hdr = open(os.path.join(ROOT, "include", "accerl.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(accerl_[a-z_0-9]+)\s*\(", hdr))
    assert {"accerl_policy_create", "accerl_actor_forward", "accerl_actor_forward_teacher",
            "accerl_actor_forward_recurrent", "accerl_actor_forward_debug", "accerl_policy_destroy",
            "accerl_last_error", "accerl_blob_sizes", "accerl_monitor_kl", "accerl_monitor_kl_noalloc", "accerl_vtrace", "accerl_distill_loss", "accerl_actor_forward_mixture", "accerl_mixture_alpha", "accerl_probe_mfma", "accerl_probe_copy", "accerl_probe_empty"} <= names
    lib = A.load_library()
    for n in names:
        assert hasattr(lib, n), n


def test_blob_sizes_match_parameter_counts(A):
    for ci, cfg in wl.CONFIGS.items():
        for role, prec in (("student", "int8"), ("teacher", cfg["teacher_precision"])):
            net = cfg[role]
            wb, ns = A.blob_sizes(A.make_arch(net, prec))
            shapes = wl.param_shapes(net)
            has_lstm = any(l["kind"] == "lstm" for l in net.layers)
            off, nsw = 0, 0
            for name, ws, bs in shapes:
                q = prec == "int8" and "lstm" not in name and not (name == "heads" and has_lstm)
                off = (off + 15) // 16 * 16 + int(np.prod(ws)) * (1 if q else 4)
                if bs is not None:
                    off = (off + 15) // 16 * 16 + int(np.prod(bs)) * 4
                nsw += ws[0] if q else 0
            assert wb == off, (ci, role)
            if prec == "int8":
                n_act = 1 + sum(1 for l in net.layers if l["kind"] in ("conv", "dense")) + \
                    2 * sum(1 for l in net.layers if l["kind"] == "resblock")
                assert ns == n_act + nsw
            else:
                assert ns == 0


def test_bad_arguments_are_rejected_before_any_gpu_work(A):
    lib = A.load_library()
    net = wl.CONFIGS[0]["student"]
    arch = A.make_arch(net, "int8")
    wb, ns = A.blob_sizes(arch)
    h = C.c_void_p()
    blob = np.zeros(wb, np.uint8)
    sc = np.ones(ns, np.float32)
    vp = lambda a: a.ctypes.data_as(C.c_void_p)
    assert lib.accerl_policy_create(None, vp(blob), wb, vp(sc), ns, C.byref(h)) == -1
    assert "NULL" in A.accerl_last_error()
    assert lib.accerl_policy_create(C.byref(arch), None, wb, vp(sc), ns, C.byref(h)) == -1
    assert lib.accerl_policy_create(C.byref(arch), vp(blob), wb - 1, vp(sc), ns, C.byref(h)) == -1
    assert lib.accerl_policy_create(C.byref(arch), vp(blob), wb, vp(sc), ns + 1, C.byref(h)) == -1
    assert lib.accerl_policy_create(C.byref(arch), vp(blob), wb, None, ns, C.byref(h)) == -1
    bad = np.ones(ns, np.float32)
    bad[1] = 0.0
    assert lib.accerl_policy_create(C.byref(arch), vp(blob), wb, vp(bad), ns, C.byref(h)) == -1
    blob128 = blob.copy()
    blob128[0] = 0x80                                    # int8 -128 is outside the symmetric range
    assert lib.accerl_policy_create(C.byref(arch), vp(blob128), wb, vp(sc), ns, C.byref(h)) == -1
    # inconsistent arch: dense input width does not match
    arch2 = A.make_arch(net, "int8")
    arch2.layers[1].cin = 63
    assert lib.accerl_blob_sizes(C.byref(arch2), None, None) == -1
    arch3 = A.make_arch(net, "int8")
    arch3.n_actions = 0
    assert lib.accerl_blob_sizes(C.byref(arch3), None, None) == -1
    # image policy without flatten before the heads
    cnn = wl.nature_cnn()
    a4 = A.make_arch(cnn, "int8")
    a4.n_layers = 3
    assert lib.accerl_blob_sizes(C.byref(a4), None, None) == -1
    # forward with a NULL policy
    assert lib.accerl_actor_forward(None, None, 4, None, None, None, None, None) == -1
    assert h.value is None


def test_product_code_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2211_15023_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith((".py", ".c")):
                assert "paper_2211_15023_amd" not in open(os.path.join(dirpath, f)).read(), f


def test_monitor_and_vtrace_reject_bad_arguments_before_any_launch(A):
    lib = A.load_library()
    # nothing below reaches the GPU: every call fails (or is a no-op) in the argument checks
    assert lib.accerl_monitor_kl(None, None, 0, 18, None, None, None, None) == 0          # B = 0: no-op
    assert lib.accerl_monitor_kl(None, None, 8, 18, None, None, None, None) == -1
    assert "NULL" in A.accerl_last_error()
    assert lib.accerl_monitor_kl(None, None, 8, 65, None, None, None, None) == -1
    assert lib.accerl_monitor_kl(None, None, -1, 4, None, None, None, None) == -1
    assert lib.accerl_vtrace(None, None, None, None, None, None, None, 0, 4, 6, 1.0, 1.0, None, None, None, None) == 0
    assert lib.accerl_vtrace(None, None, None, None, None, None, None, 4, 4, 6, 1.0, 1.0, None, None, None, None) == -1
    assert lib.accerl_vtrace(None, None, None, None, None, None, None, 4, 4, 0, 1.0, 1.0, None, None, None, None) == -1
    assert lib.accerl_vtrace(None, None, None, None, None, None, None, 4, 4, 6, -1.0, 1.0, None, None, None, None) == -1


def _plan(A, net, prec, tensors, scales=None):
    blob = A.pack_weights(tensors)
    sc = A.pack_scales(scales, tensors) if scales is not None else None
    return A.accerl_plan_describe(A.make_arch(net, prec), blob, sc)


def _fields(line):
    return dict(tok.split("=", 1) for tok in line.split() if "=" in tok)


def test_planner_decisions_on_the_benchmark_networks(A):
    """Host-only view of the launch plans: the fusions and layouts the kernels rely on are chosen where expected."""
    from helpers import policies
    # config 2 student: first two convs share a kernel; conv3 runs wave-private
    nt, pt, ns, ps, qp = policies(2, 8)
    steps = [l for l in _plan(A, ns, "int8", qp.tensors, qp.act_scales).splitlines() if l.startswith("step")]
    convs = [_fields(l) for l in steps if " conv " in l]
    assert [c["fuse_next"] for c in convs] == ["1", "0", "0"]
    assert convs[0]["mode"] == "2" and convs[0]["KS"] == "4" and convs[2]["wp"] == "1"
    # the paper's original network gets the kernels with compile-time sizes, and its last convolution hands the
    # dense layer its input in MFMA fragment order
    assert [c["front"] for c in convs] == ["1", "0", "0"] and [c["tail"] for c in convs] == ["0", "0", "1"]
    assert [c["out_frag"] for c in convs] == ["0", "0", "1"]
    # with these weights no input can drive an accumulator of the three layers to 2^23: three-instruction requantization
    assert [c["pos23"] for c in convs] == ["1", "1", "1"]
    gemms = [_fields(l) for l in steps if " gemm " in l]
    assert gemms[0]["x_frag"] == "1" and gemms[0]["k_steps"] == "49"
    # the paper's smaller students (16 and 32 filters): layer by layer, and 9 * 9 * 32 bytes are not whole MFMA steps,
    # so the dense layer reads plain rows
    from workloads.configs import PAPER_STUDENTS
    import oracle
    net = PAPER_STUDENTS["net1"]
    params = wl.init_params(net, wl.STREAM["weights_student"])
    q1 = oracle.quantize_policy(net, params, wl.make_frames_u8(8, stream=wl.STREAM["calibration"]))
    s1 = [l for l in _plan(A, net, "int8", q1.tensors, q1.act_scales).splitlines() if l.startswith("step")]
    c1 = [_fields(l) for l in s1 if " conv " in l]
    assert [c["front"] for c in c1] == ["0", "0"] and [c["tail"] for c in c1] == ["0", "0"]
    assert all(c["out_frag"] == "0" for c in c1) and all(_fields(l)["x_frag"] == "0" for l in s1 if " gemm " in l)
    # config 3 student: thin layers are pixel-packed (8 stored channels -> 16-row tiles at half the width),
    # the three stack convs carry their max-pool, residual convs do not
    nt, pt, ns, ps, qp = policies(3, 8)
    steps = [l for l in _plan(A, ns, "int8", qp.tensors, qp.act_scales).splitlines() if l.startswith("step")]
    convs = [_fields(l) for l in steps if " conv " in l]
    assert convs[0]["out"] == "84x42x16" and convs[1]["out"] == "42x21x16"
    assert [c["pool"] for c in convs].count("1") == 3 and convs[0]["pool"] == "1"
    assert all(int(c["PF"]) <= 4 for c in convs)                   # small batches: four workgroups per compute unit
    assert sum(1 for l in steps if " maxpool " in l) == 3          # kept in the plan for debug taps
    # every residual block of the student is one launch: its first convolution carries the second
    assert [c["resblock"] for c in convs] == ["0", "1", "0", "1", "0", "0", "1", "0", "1", "0", "0", "1", "0", "1", "0"]
    assert [c["fuse_next"] for c in convs] == [c["resblock"] for c in convs]
    # and every stack (conv + pool + two blocks) is one launch: the stack convolution heads it, the four block
    # convolutions behind it are its members; 5 launches remain (three stacks, the dense layer, the heads)
    assert [c["stack"] for c in convs] == ["1", "2", "2", "2", "2"] * 3
    # the stack convolutions have no ReLU before their max-pool, so the offset accumulators are not for them
    assert [c["pos23"] for c in convs][0] == "0" and convs[1]["pos23"] == "1"
    # the teacher's wider layers are not packed
    tsteps = [l for l in _plan(A, nt, "bf16", [dict(w=w, b=b) for _, w, b in pt]).splitlines() if l.startswith("step")]
    assert _fields([l for l in tsteps if " conv " in l][0])["out"] == "84x84x16"
    assert all(_fields(l)["resblock"] == "0" and _fields(l)["stack"] == "0" for l in tsteps if " conv " in l)   # bf16 blocks run layer by layer


def test_workspace_slots_are_shared(A):
    from helpers import policies
    nt, pt, ns, ps, qp = policies(3, 8)
    head = _plan(A, ns, "int8", qp.tensors, qp.act_scales).splitlines()[0]
    per_state = int(_fields(head)["ws_bytes_per_state"])
    shapes = wl.trace_shapes(ns)
    naive = sum(int(np.prod(s)) for s in shapes if len(s) == 3)    # one buffer per image-shaped layer output
    assert per_state < naive / 3
    # with whole stacks fused only the stack outputs and the dense layer's output need workspace, and the third stack's
    # and the dense layer's share the slot the first stack's output has left
    assert per_state == 42 * 42 * 8 + 21 * 21 * 16
