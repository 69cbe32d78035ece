#!/usr/bin/env python3
"""Benchmark of the actor forward on one MI355X.

A "step" is one accerl_actor_forward call of the int8 student over one batch of synthetic Atari-like
frames already resident in HBM (Nature-DQN CNN, B = 4096: the network the paper's own "Original"
row and its 6 ms -> 3 ms int8 figure refer to).  `value` is states per second of that call.  The
same line carries: the B = 160 forward latency (the paper's batch size), the bf16 teacher's numbers
and the student/teacher speedup, the per-kernel breakdown, the roofline figure of the dominant
kernel (HIP events around every launch, in a second pass over the same steps), and the CPU oracle
timed on this machine's host cores on a sample of the same states.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--batch 4096]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"int8": 5.0e15, "bf16": 2.5e15, "fp32": 157.3e12, "hbm": 8.0e12}


def layer_macs(net, shapes_in):
    """Useful multiply-accumulates per state of each parametrised layer, keyed by arch layer index
    (resblock: both convolutions; n_layers: the heads)."""
    import workloads as wl
    out = {}
    shp = tuple(net.obs_shape)
    outs = wl.trace_shapes(net)
    for i, L in enumerate(net.layers):
        o = outs[i]
        if L["kind"] == "conv":
            out[i] = o[1] * o[2] * L["cout"] * L["cin"] * L["k"] ** 2
        elif L["kind"] == "resblock":
            out[i] = 2 * o[1] * o[2] * L["ch"] * L["ch"] * 9
        elif L["kind"] == "dense":
            out[i] = L["cin"] * L["cout"]
        elif L["kind"] == "lstm":
            out[i] = 4 * L["hidden"] * (L["cin"] + L["hidden"])
        shp = o
    out[len(net.layers)] = (net.n_actions + 1) * wl.feature_dim(net)
    return out


def io_bytes(net):
    """Algorithmic HBM bytes per state: observation in, uniform in, logits / value / action out."""
    import numpy as np
    obs = int(np.prod(net.obs_shape)) * (1 if net.obs_dtype == "u8" else 4)
    return obs + 4 + net.n_actions * 4 + 4 + 4


def kernel_source_hash():
    """sha256 over the kernel sources: a counter summary under profiles/ quotes the hash of the sources it was measured
    on, and is only used while it still matches."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2211_15023_amd", "csrc", "*"))):
        if f.endswith((".hip", ".h")):
            h.update(os.path.basename(f).encode())
            h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def time_forward(pol, x, u, outs, steps, warmup, **kw):
    import torch
    for _ in range(warmup):
        pol.forward(x, u, outputs=outs, **kw)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        pol.forward(x, u, outputs=outs, **kw)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the first milliseconds after an idle period run at lower clocks (a forward of the default workload takes 73 us
    # over 50 steps, 61 us from about 2000 steps on): the defaults measure the sustained rate, in a fraction of a second
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-extra", action="store_true", help="only the headline workload")
    ap.add_argument("--no-per-config", action="store_true", help="skip the table of all five configurations")
    ap.add_argument("--paper-nets", action="store_true",
                    help="also time the paper's own networks (network table: Original with FC 2048, Net1-Net3)")
    ap.add_argument("--ceilings", action="store_true",
                    help="also measure what this machine sustains: register-resident MFMA loops and a streaming copy")
    ap.add_argument("--copy-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (a known-size reference for HBM counters)")
    ap.add_argument("--source-hash", action="store_true", help="print the hash of the kernel sources and exit")
    args = ap.parse_args()
    if args.source_hash:
        print(kernel_source_hash())
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU only (states are independent rows; a fleet of actors "
              "shards by row with no exchange on the forward path). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as wl
    import paper_2211_15023_amd as A
    # Post-training quantization and pruning are the Compressor's offline step (Section 2.2), outside the library:
    # the oracle's host helper produces the policy bytes, exactly as the parity tests do, so that the timed policy
    # is the one the oracle is compared with.
    import oracle

    A.load_library()
    ci = args.config
    cfg = wl.CONFIGS[ci]
    nt, ns = cfg["teacher"], cfg["student"]
    B = args.batch or (cfg["batches"][1] if ci == 2 else cfg["batches"][-1])
    tprec = cfg["teacher_precision"]

    def states(net, n, stream):
        if net.obs_dtype == "u8":
            return wl.make_frames_u8(n, *net.obs_shape, stream=stream)
        return wl.make_obs_f32(n, net.obs_shape[0], stream=stream)

    # ---- policies (Compressor output on the host, once)
    pt = wl.init_params(nt, wl.STREAM["weights_teacher"])
    if cfg["student_from"] == "quantize":
        ps = pt
    elif cfg["student_from"] == "independent":
        ps = wl.init_params(ns, wl.STREAM["weights_student"])
    else:
        ps, _ = oracle.prune_policy(nt, pt, ns)
    qp = oracle.quantize_policy(ns, ps, states(ns, cfg["calib"], wl.STREAM["calibration"]))
    tensors, act_scales = qp.tensors, qp.act_scales
    teacher_tensors = lambda params: [dict(name=n, w=w, b=b) for n, w, b in params]
    student = A.Policy(ns, "int8", tensors, act_scales)
    teacher = A.Policy(nt, tprec, teacher_tensors(pt))

    # ---- inputs, resident in HBM before any timed region
    x_host = states(ns, B, wl.STREAM["states"])
    u_host = wl.make_uniforms(B)
    x, u = torch.from_numpy(x_host).cuda(), torch.from_numpy(u_host).cuda()
    kw = {}
    if student.recurrent:
        h, c = wl.make_hc(B, 256)
        kw = dict(done=torch.from_numpy(wl.make_done(1, B)[0]).cuda(), h=torch.from_numpy(h).cuda(), c=torch.from_numpy(c).cuda())
    outs = student.alloc_outputs(B)
    torch.cuda.synchronize()

    if args.copy_mb:
        src = torch.empty(args.copy_mb << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()

    # ---- headline: K timed steps of the student
    sec = time_forward(student, x, u, outs, args.steps, args.warmup, **kw)
    value = B / sec

    # ---- second pass with HIP events around every launch: per-kernel breakdown and roofline
    A.accerl_profile_begin(student.handle)
    for _ in range(args.steps):
        student.forward(x, u, outputs=outs, **kw)
    torch.cuda.synchronize()
    prof = A.accerl_profile_end(student.handle)
    macs = layer_macs(ns, None)
    n_launch_step = sum(p["launches"] for p in prof) / args.steps
    breakdown = []
    def step_macs(p):
        m = macs.get(p["layer"], 0) if p["kind"] in ("conv", "gemm", "heads") else 0
        if p["layer"] < len(ns.layers) and ns.layers[p["layer"]]["kind"] == "resblock":
            m //= 2
        return m
    for p in prof:
        if not p["launches"]:
            # a conv or max-pool done inside the kernel of the step before it: its work counts there
            if breakdown and p["kind"] in ("conv", "maxpool"):
                breakdown[-1]["layers"].append(p["layer"])
                breakdown[-1]["macs"] += step_macs(p)
            continue
        per_step_ms = p["total_ms"] / args.steps
        breakdown.append(dict(step=p["step"], kind=p["kind"], layer=p["layer"], layers=[p["layer"]], macs=step_macs(p),
                              ms_per_step=round(per_step_ms, 5), launches_per_step=p["launches"] / args.steps))
    for ent in breakdown:
        if ent["macs"]:
            ent["tops"] = round(2 * ent["macs"] * B / (ent["ms_per_step"] * 1e-3) / 1e12, 2)
    dom = max(breakdown, key=lambda e: e["ms_per_step"])
    launches = dom["launches_per_step"]
    span_s = dom["ms_per_step"] * 1e-3 / launches
    # An event after every launch makes the step slower than the timed steps were: the difference, shared equally
    # among the launches, is what an event costs (about 2.5 us each); a span less that share is the kernel plus
    # its launch gap as it runs in the timed region, and what rocprofv3's kernel duration is to be compared with.
    event_s = max(0.0, (sum(e["ms_per_step"] for e in breakdown) * 1e-3 - sec) / n_launch_step)
    avg_launch_s = span_s - event_s
    obs_bytes = int(np.prod(ns.obs_shape)) * (1 if ns.obs_dtype == "u8" else 4)
    first_param = min(macs) if macs else -1
    if dom["kind"] in ("conv", "gemm", "heads"):
        m = dom["macs"]
        is_bf16 = student.recurrent and dom["layer"] >= len(ns.layers) - 1
        ops_launch = 2.0 * m * B / launches
        peak = PEAK["bf16" if is_bf16 else "int8"]
        t_mfma = ops_launch / peak
        t_hbm = obs_bytes * B / launches / PEAK["hbm"] if dom["layer"] == first_param else 0.0
        if t_hbm > t_mfma:
            # the kernel that reads the observations: its algorithmic bytes (the observation, read once)
            # take longer at HBM peak than its multiply-accumulates at MFMA peak
            bytes_launch = obs_bytes * B / launches
            roofline = dict(bound="hbm", achieved=round(bytes_launch / avg_launch_s / 1e9, 2), peak=PEAK["hbm"] / 1e9,
                            unit="GB/s", frac=round(bytes_launch / avg_launch_s / PEAK["hbm"], 4), traffic=None,
                            kernel=f"{dom['kind']} layers {dom['layers']}", avg_launch_us=round(avg_launch_s * 1e6, 2),
                            launches_per_step=launches, mfma_frac=round(ops_launch / avg_launch_s / peak, 4))
        else:
            roofline = dict(bound="mfma", achieved=round(ops_launch / avg_launch_s / 1e12, 3), peak=peak / 1e12,
                            unit="TFLOP/s", frac=round(ops_launch / avg_launch_s / peak, 4), traffic=None,
                            kernel=f"{dom['kind']} layers {dom['layers']}", avg_launch_us=round(avg_launch_s * 1e6, 2),
                            launches_per_step=launches)
    else:
        bytes_launch = io_bytes(ns) * B / launches
        roofline = dict(bound="hbm", achieved=round(bytes_launch / avg_launch_s / 1e9, 2), peak=PEAK["hbm"] / 1e9,
                        unit="GB/s", frac=round(bytes_launch / avg_launch_s / PEAK["hbm"], 4), traffic=None,
                        kernel=f"{dom['kind']} layers {dom['layers']}", avg_launch_us=round(avg_launch_s * 1e6, 2),
                        launches_per_step=launches)
    roofline["event_span_us"] = round(span_s * 1e6, 2)
    roofline["event_cost_us"] = round(event_s * 1e6, 2)
    # HBM bytes per launch of that kernel from the committed counter summary, if it was measured on these very sources
    tfile = os.path.join(ROOT, "profiles", f"traffic_cfg{ci}_B{B}.txt")
    roofline["traffic_note"] = "no counter summary for this workload"
    if os.path.exists(tfile):
        kv = dict(l.strip().split("=", 1) for l in open(tfile) if "=" in l and not l.startswith("#"))
        if kv.get("kernel_source_hash") == kernel_source_hash():
            roofline["traffic"] = float(kv["traffic_bytes_per_launch"])
            roofline["traffic_note"] = "FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 from " + os.path.basename(tfile)
        else:
            roofline["traffic_note"] = ("stale: " + os.path.basename(tfile) + " was measured on other kernel sources (hash " +
                                        str(kv.get("kernel_source_hash")) + ", now " + kernel_source_hash() + ")")

    total_macs = sum(macs.values())
    whole = dict(useful_tops=round(2 * total_macs * B / sec / 1e12, 2), frac_int8_peak=round(2 * total_macs * B / sec / PEAK["int8"], 4),
                 io_gbps=round(io_bytes(ns) * B / sec / 1e9, 2), frac_hbm_peak=round(io_bytes(ns) * B / sec / PEAK["hbm"], 4))

    extra = dict(kernels=breakdown, whole_forward=whole, launches_per_step=n_launch_step)
    if not args.no_extra:
        # teacher at the same batch, and both at the paper's batch size of 160
        touts = teacher.alloc_outputs(B)
        xt = x if nt.obs_dtype == ns.obs_dtype and nt.obs_shape == ns.obs_shape else torch.from_numpy(states(nt, B, wl.STREAM["states"])).cuda()
        tsec = time_forward(teacher, xt, u, touts, max(5, args.steps // 4), max(3, args.warmup // 4), **kw)
        extra["teacher"] = dict(precision=tprec, states_per_s=round(B / tsec, 1), ms_per_step=round(tsec * 1e3, 4))
        extra["student_over_teacher"] = round(tsec / sec, 3)
        b160 = min(160, B)
        o160 = student.alloc_outputs(b160)
        kw160 = {k: v[:b160].contiguous() for k, v in kw.items()}
        s160 = time_forward(student, x[:b160].contiguous(), u[:b160].contiguous(), o160, 2000, 200, **kw160)
        t160 = time_forward(teacher, xt[:b160].contiguous(), u[:b160].contiguous(), teacher.alloc_outputs(b160), 1000, 100, **kw160)
        extra["latency_B160_us"] = dict(student=round(s160 * 1e6, 2), teacher=round(t160 * 1e6, 2))
        # what a launch costs on this machine: chains of a kernel that does nothing, back to back on the same stream,
        # timed like the forwards (host clock around 2000 launches) -- the floor under the latency of the small batches
        for _ in range(200):
            A.accerl_probe_empty()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(2000):
            A.accerl_probe_empty()
        torch.cuda.synchronize()
        floor = (time.perf_counter() - t0) / 2000
        n_l = int(round(n_launch_step))
        extra["launch_floor_us"] = dict(one_empty_launch=round(floor * 1e6, 2), launches_per_forward=n_l,
                                        floor_per_forward=round(floor * n_l * 1e6, 2),
                                        student_B160_over_floor=round(s160 / (floor * n_l), 2))

        # spread of the per-call time: 200 chains of 10 back-to-back calls, an event before and after each chain
        # (both on the stream the kernels run on), p10 / median / p90 of chain time / 10
        def spread(pol, xs, us, o, **kws):
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
            for _ in range(200):
                pol.forward(xs, us, outputs=o, **kws)
            for a, b in evs:
                a.record()
                for _ in range(10):
                    pol.forward(xs, us, outputs=o, **kws)
                b.record()
            torch.cuda.synchronize()
            t = np.sort(np.array([a.elapsed_time(b) for a, b in evs])) * 100.0      # ms per chain -> us per call
            return dict(p10=round(float(t[20]), 2), p50=round(float(t[100]), 2), p90=round(float(t[180]), 2))
        extra["per_call_us_spread"] = dict(student=spread(student, x, u, outs, **kw),
                                           student_B160=spread(student, x[:b160].contiguous(), u[:b160].contiguous(), o160, **kw160))
        # two Actors on one GPU (Actor section: several actor threads share an accelerator): a second policy object with
        # its own workspace and stream, forwards issued alternately; one batch fills while the other drains
        if not student.recurrent:
            second = A.Policy(ns, "int8", tensors, act_scales)
            pair = [(student, outs, torch.cuda.Stream()), (second, second.alloc_outputs(B), torch.cuda.Stream())]
            torch.cuda.synchronize()

            def alternate(n):
                for i in range(n):
                    pol, o, st = pair[i & 1]
                    pol.forward(x, u, outputs=o, stream=st)
                torch.cuda.synchronize()
            alternate(2 * args.warmup)
            t0 = time.perf_counter()
            alternate(2 * args.steps)
            t2 = (time.perf_counter() - t0) / (2 * args.steps)
            extra["two_actor_streams"] = dict(states_per_s=round(B / t2, 1), ms_per_step=round(t2 * 1e3, 5))
            second.close()
        # the two consumers of the behaviour logits, on one unroll of 16 steps x B environments
        # (Monitor section, KL equation; Corrector section, V-trace equation); both HBM-bound
        nA = ns.n_actions

        def timed(fn, n=50):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / n
        for Tn, tag in ((16, ""), (256, "_long")):      # one unroll as configured; a long one where launch cost fades
            tr = wl.make_trajectory(Tn, B, nA)
            dv = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in tr.items()}
            rows = Tn * B
            klo = torch.empty(rows, dtype=torch.float32, device="cuda")
            eno = torch.empty_like(klo)
            sto = torch.zeros(4, dtype=torch.float64, device="cuda")
            lo2, ls2 = dv["logits_original"].view(rows, nA), dv["logits_smaller"].view(rows, nA)
            vso = torch.empty(Tn, B, dtype=torch.float32, device="cuda")
            ado, rho = torch.empty_like(vso), torch.empty_like(vso)
            t_kl = timed(lambda: A.accerl_monitor_kl(lo2, ls2, klo, eno, sto))
            t_vt = timed(lambda: A.accerl_vtrace(dv["logits_original"], dv["logits_smaller"], dv["actions"], dv["rewards"],
                                                dv["discounts"], dv["values"], dv["bootstrap"], 1.0, 1.0, vso, ado, rho))
            kl_bytes = rows * (2 * nA * 4 + 8)                         # both logit rows in, KL and entropy out
            vt_bytes = rows * (2 * nA * 4 + 4 + 4) + rows * (4 * 4 + 3 * 4) + B * 4   # ratio pass + scan pass
            extra["monitor_kl" + tag] = dict(rows=rows, actions=nA, us=round(t_kl * 1e6, 2), gbps=round(kl_bytes / t_kl / 1e9, 1),
                                             frac_hbm_peak=round(kl_bytes / t_kl / PEAK["hbm"], 4))
            extra["vtrace" + tag] = dict(T=Tn, B=B, actions=nA, us=round(t_vt * 1e6, 2), gbps=round(vt_bytes / t_vt / 1e9, 1),
                                         frac_hbm_peak=round(vt_bytes / t_vt / PEAK["hbm"], 4))

    if not args.no_extra and not args.no_per_config:
        # every configuration at its largest configured batch: student and teacher time per forward and their ratio
        # (the student / teacher speedup the paper reports for its compressed actors), with the share of the int8 MFMA
        # peak (useful operations) and of the HBM peak (observations + outputs) that the student reaches
        per = {}
        frames = None
        for cj, cfg_j in wl.CONFIGS.items():
            ntj, nsj = cfg_j["teacher"], cfg_j["student"]
            Bj = cfg_j["batches"][-1]
            ptj = wl.init_params(ntj, wl.STREAM["weights_teacher"])
            if cfg_j["student_from"] == "quantize":
                psj = ptj
            elif cfg_j["student_from"] == "independent":
                psj = wl.init_params(nsj, wl.STREAM["weights_student"])
            else:
                psj, _ = oracle.prune_policy(ntj, ptj, nsj)
            qpj = oracle.quantize_policy(nsj, psj, states(nsj, cfg_j["calib"], wl.STREAM["calibration"]))
            stu_j = A.Policy(nsj, "int8", qpj.tensors, qpj.act_scales)
            tea_j = A.Policy(ntj, cfg_j["teacher_precision"], teacher_tensors(ptj))
            if nsj.obs_dtype == "u8":
                if frames is None or frames.shape[0] < Bj:
                    frames = torch.from_numpy(states(nsj, max(Bj, 16384), wl.STREAM["states"])).cuda()
                xj = frames[:Bj].contiguous()
            else:
                xj = torch.from_numpy(states(nsj, Bj, wl.STREAM["states"])).cuda()
            uj = torch.from_numpy(wl.make_uniforms(Bj)).cuda()
            kwj = {}
            if stu_j.recurrent:
                hj, cj2 = wl.make_hc(Bj, 256)
                kwj = dict(done=torch.from_numpy(wl.make_done(1, Bj)[0]).cuda(), h=torch.from_numpy(hj).cuda(), c=torch.from_numpy(cj2).cuda())
            n_s = 400 if Bj * sum(layer_macs(nsj, None).values()) < 1e11 else 60
            ts = time_forward(stu_j, xj, uj, stu_j.alloc_outputs(Bj), n_s, max(5, n_s // 10), **kwj)
            tt = time_forward(tea_j, xj, uj, tea_j.alloc_outputs(Bj), max(5, n_s // 8), 3, **kwj)
            mj = sum(layer_macs(nsj, None).values())
            per[f"config{cj}_{cfg_j['name']}"] = dict(
                B=Bj, student_us=round(ts * 1e6, 2), teacher_us=round(tt * 1e6, 2), teacher_precision=cfg_j["teacher_precision"],
                student_states_per_s=round(Bj / ts, 1), student_over_teacher=round(tt / ts, 2),
                frac_int8_peak=round(2 * mj * Bj / ts / PEAK["int8"], 4), frac_hbm_peak=round(io_bytes(nsj) * Bj / ts / PEAK["hbm"], 4))
            # the student's latency at every configured batch of this configuration
            by_b = {}
            for bb in cfg_j["batches"]:
                kwb = {k: v[:bb].contiguous() for k, v in kwj.items()}
                tb = time_forward(stu_j, xj[:bb].contiguous(), uj[:bb].contiguous(), stu_j.alloc_outputs(bb), 300 if bb <= 1024 else n_s, 30, **kwb)
                by_b[str(bb)] = round(tb * 1e6, 2)
            per[f"config{cj}_{cfg_j['name']}"]["student_us_by_batch"] = by_b
            if stu_j.recurrent and "unroll" in cfg_j:
                # the configured unroll as an actor runs it: one call per environment step, the state carried in place
                # (the observations of all steps are resident, as the workload states; done flags ~ Bernoulli(0.01))
                Tn = cfg_j["unroll"]
                dn = torch.from_numpy(wl.make_done(Tn, Bj)).cuda()
                outs_j = stu_j.alloc_outputs(Bj)
                def unroll():
                    for t in range(Tn):
                        stu_j.forward(xj, uj, outputs=outs_j, done=dn[t], h=kwj["h"], c=kwj["c"])
                for _ in range(3):
                    unroll()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(10):
                    unroll()
                torch.cuda.synchronize()
                tu = (time.perf_counter() - t0) / 10
                per[f"config{cj}_{cfg_j['name']}"].update(unroll_steps=Tn, unroll_ms=round(tu * 1e3, 3),
                                                          unroll_state_steps_per_s=round(Tn * Bj / tu, 1))
            stu_j.close()
            tea_j.close()
        del frames
        extra["per_config"] = per

    if args.ceilings:
        def span(fn, n=60):
            for _ in range(10):          # clocks up before the timed launches
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / n
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        iters = 4000
        waves = 2048 * 4
        t_i8 = span(lambda: A.accerl_probe_mfma(0, iters, sink))
        t_bf = span(lambda: A.accerl_probe_mfma(1, iters, sink))
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(3)
        dst = torch.empty_like(src)
        t_cp = span(lambda: A.accerl_probe_copy(src, dst))
        extra["ceilings"] = dict(int8_mfma_tops=round(waves * iters * 8 * 2 * 16 * 16 * 64 / t_i8 / 1e12, 1),
                                 bf16_mfma_tflops=round(waves * iters * 8 * 2 * 16 * 16 * 32 / t_bf / 1e12, 1),
                                 copy_1gib_read_plus_write_gbps=round(2 * (1 << 30) / t_cp / 1e9, 1))
        del src, dst

    if args.paper_nets:
        # the networks of the paper's table (Section 3.1), each as int8 and bf16, at the paper's batch of 160
        # and at the benchmark batch; weights seeded, int8 scales calibrated on 64 seeded states
        table = {}
        nets = [("original_fc2048", wl.nature_cnn("original_fc2048", fc=2048))] + list(wl.configs.PAPER_STUDENTS.items())
        for name, net in nets:
            params = wl.init_params(net, wl.STREAM["weights_student"])
            qn = oracle.quantize_policy(net, params, states(net, 64, wl.STREAM["calibration"]))
            pols = dict(int8=A.Policy(net, "int8", qn.tensors, qn.act_scales), bf16=A.Policy(net, "bf16", teacher_tensors(params)))
            row = {}
            for bb in (160, B):
                xb, ub = x[:bb].contiguous(), u[:bb].contiguous()
                for prec, pol in pols.items():
                    t = time_forward(pol, xb, ub, pol.alloc_outputs(bb), 1000, 100)
                    row[f"{prec}_B{bb}_us"] = round(t * 1e6, 2)
            for pol in pols.values():
                pol.close()
            table[name] = row
        extra["paper_nets"] = table

    # ---- the CPU oracle on a sample of the same states (rank 0, N = 1 only)
    cpu = None
    if not args.no_cpu:
        from oracle import layers as OL
        nsamp = {0: B, 1: B, 2: 4096, 3: 2048, 4: 2048}.get(ci, 256)
        nsamp = min(nsamp, B)
        okw = {}
        if student.recurrent:
            hh, cc = wl.make_hc(B, 256)
            okw = dict(h=hh[:nsamp], c=cc[:nsamp], done=wl.make_done(1, B)[0][:nsamp])
        reps = 1
        oracle.forward_int8(ns, qp, x_host[:min(nsamp, 8)], u_host[:min(nsamp, 8)], **{k: v[:min(nsamp, 8)] for k, v in okw.items()})
        t0 = time.perf_counter()
        ref = oracle.forward_int8(ns, qp, x_host[:nsamp], u_host[:nsamp], **okw)
        dt = time.perf_counter() - t0
        while dt * reps < 4.0 and reps < 4096:       # small networks: repeat to get a stable figure
            reps *= 4
            t0 = time.perf_counter()
            for _ in range(reps):
                oracle.forward_int8(ns, qp, x_host[:nsamp], u_host[:nsamp], **okw)
            dt = (time.perf_counter() - t0) / reps
        cpu = dict(value=round(nsamp / dt, 1), unit="states/s", cores=OL.num_threads(), kind="oracle",
                   sample=f"first {nsamp} of the {B} benchmark states, int8 student, {dt:.2f} s per pass")
        # the same oracle on one thread, on a prefix sized for a few seconds
        n1 = max(1, min(nsamp, int(nsamp / dt * 3.0 / max(1, OL.num_threads()))))
        all_threads = OL.num_threads()
        OL.set_threads(1)
        try:
            t0 = time.perf_counter()
            oracle.forward_int8(ns, qp, x_host[:n1], u_host[:n1], **{k: v[:n1] for k, v in okw.items()})
            d1 = time.perf_counter() - t0
        finally:
            OL.set_threads(all_threads)
        cpu["single_thread"] = dict(value=round(n1 / d1, 1), unit="states/s", cores=1,
                                    sample=f"first {n1} states, {d1:.2f} s")
        # the same sample doubles as an end-of-run parity check of the timed configuration
        got = outs[0][:nsamp].cpu().numpy()
        extra["parity_sample_logits_equal"] = bool(np.array_equal(got, ref["logits"])) if not student.recurrent else None

    line = {
        "metric": "actor states/sec (int8 student vs fp32/bf16 teacher); B=160 forward latency",
        "value": round(value, 1), "unit": "states/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config {ci} ({cfg['name']}): int8 student {ns.name}, B={B}, "
                               f"obs {ns.obs_dtype}{list(ns.obs_shape)}, {ns.n_actions} actions", "batch": B},
        "roofline": roofline, "cpu_baseline": cpu, "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
