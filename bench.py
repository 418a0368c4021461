#!/usr/bin/env python3
"""Benchmark of the dual-scale W8A8 linear on one MI355X.

A "step" is one pass of the online hot path (activation quantization with the gather-permute,
then the dual INT8 GEMM with its dequant epilogue) over every layer of the workload.  The headline
workload is config 2: the six linears of a Wan-1.3B-style DiT block for one 3-latent-frame chunk
(M = 4680 tokens), each at the four planted outlier counts {0, 4, 16, 64} -- 24 layers, 48 kernel
launches on one stream.  The offline weight step (detection, permutation, dual scales) runs once
before the timed region.  All inputs are resident in HBM when timing starts.

Prints ONE JSON line.  `value` = sum over layers of 2*M*N*K divided by the step time (INT8 TOPS of
the whole linear, quantization included) on config 2.  Also in the line:
  roofline / quant_act_roofline   the GEMM at the target shape (M=4680, 1536 -> 8960) against the dense
                                  INT8 MFMA peak and the activation kernel against the HBM peak, both from
                                  per-launch HIP events inside the step ("in-step": operands evicted by the
                                  other layers);
  layers                          per layer: in-step and back-to-back times of both kernels, the bf16
                                  torch.nn.functional.linear comparator timed the same two ways;
  configs                         the other four workloads, compact (per distinct shape);
  cpu_baseline                    the CPU oracle on a bounded sample, host threads stated.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0      # MI355X dense INT8 MFMA, published
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="headline workload config (2 = the one the metric is quoted on)")
    ap.add_argument("--layers", type=str, default="", help="comma-separated layer names to restrict the step to")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bf16", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the side measurements (W4A8, chained FFN, fused QKV)")
    ap.add_argument("--other-configs", type=str, default="1,3,4,5",
                    help="configs reported compactly beside the headline ('' = none)")
    ap.add_argument("--variant", type=int, default=0, help="GEMM kernel variant (0 = heuristic)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a 256 MiB device-to-device copy (reference dispatch for scaling the HBM traffic counters)")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (token rows would shard across GPUs with no exchange step); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2605_21072_amd as q
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    q.load_library()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    F = torch.nn.functional
    if args.copy_calibration:
        a = torch.full((256 << 20,), 3, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": int(a.numel())}))
        return

    def event():
        return torch.cuda.Event(enable_timing=True)

    # ---- building a workload: synthetic tensors -> HBM, weight step once per layer ----------
    def build_layers(specs, with_bf16):
        layers = []
        for s in specs:
            L = wl.make_layer(s)
            W = torch.from_numpy(L["W"]).to(dev)
            w = q.quantize_weight(W, want_norms=False)
            X = torch.from_numpy(L["X"]).to(dev)
            layer = dict(spec=s, w=w, X=X, bias=torch.from_numpy(L["bias"]).to(dev),
                         perm=w.perm if w.K_o > 0 else None,
                         Xq=torch.empty((s.M, q.packed_ld(s.K, w.K_o)), dtype=torch.int8, device=dev),
                         sx=torch.empty(s.M, dtype=torch.float32, device=dev),
                         Y=torch.empty((s.M, s.N), dtype=torch.bfloat16, device=dev))
            if with_bf16:
                layer["Wb"] = W.to(torch.bfloat16)
                layer["Xb"] = X.to(torch.bfloat16)
                layer["bb"] = layer["bias"].to(torch.bfloat16)
            del W, L
            layers.append(layer)
        torch.cuda.synchronize()
        return layers

    def run_quant(l):
        q.quant_act(l["X"], l["perm"], l["w"].K_o, Xq=l["Xq"], s_x=l["sx"])

    def run_gemm(l):
        q.w8a8_dual_gemm(l["Xq"], l["sx"], l["w"], l["bias"], l["spec"].M, Y=l["Y"], variant=args.variant)

    def run_bf16(l):
        F.linear(l["Xb"], l["Wb"], l["bb"])

    def timed_steps(layers, steps, warmup):
        """W warm-up steps, then exactly K steps between synchronisations; ms per step."""
        def step():
            for l in layers:
                run_quant(l)
                run_gemm(l)
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / steps

    def instrumented(layers, steps, fns):
        """The same steps with an event after every launch: average microseconds per launch, [len(fns)][layers]."""
        nl, nf = len(layers), len(fns)
        ev = [[event() for _ in range(nf * nl + 1)] for _ in range(steps)]
        for s_i in range(steps):
            ev[s_i][0].record()
            for i, l in enumerate(layers):
                for f_i, fn in enumerate(fns):
                    fn(l)
                    ev[s_i][nf * i + f_i + 1].record()
        torch.cuda.synchronize()
        us = np.zeros((nf, nl))
        for s_i in range(steps):
            for i in range(nl):
                for f_i in range(nf):
                    us[f_i][i] += 1e3 * ev[s_i][nf * i + f_i].elapsed_time(ev[s_i][nf * i + f_i + 1])
        return us / steps

    def back_to_back(fn, l, reps):
        """One launch repeated on the same operands between one pair of events (warm caches)."""
        for _ in range(3):
            fn(l)
        e0, e1 = event(), event()
        e0.record()
        for _ in range(reps):
            fn(l)
        e1.record()
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / reps

    def rotating(fn, group, reps):
        """One kernel launched back to back over the layers of `group` in turn (each launch finds its operands
        evicted when the group's inputs total more than the 256 MB last-level cache): microseconds per launch."""
        for l in group:
            fn(l)
        e0, e1 = event(), event()
        e0.record()
        for _ in range(reps):
            for l in group:
                fn(l)
        e1.record()
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / (reps * len(group))

    # ======================================================================= headline workload
    specs = wl.config_layers(args.config)
    if args.layers:
        keep = set(args.layers.split(","))
        specs = [s for s in specs if s.name in keep]
    assert specs, "no layers selected"
    layers = build_layers(specs, not args.no_bf16)
    nl = len(layers)

    ms_per_step = timed_steps(layers, args.steps, args.warmup)
    total_ops = sum(2.0 * l["spec"].macs for l in layers)
    value = total_ops / (ms_per_step * 1e-3) / 1e12

    quant_us, gemm_us = instrumented(layers, args.steps, [run_quant, run_gemm])

    def run_linear(l):
        run_quant(l)
        run_gemm(l)
    # the whole linear between one pair of events per LAYER: the bf16 comparator's step also carries one event per
    # layer, so this, not quant_us + gemm_us (two events), is what speedup_linear_vs_bf16 compares with
    linear_us = instrumented(layers, args.steps, [run_linear])[0]
    # what the per-launch events add: the instrumented pass against the plain timed pass, per launch
    event_overhead_us = (float(quant_us.sum() + gemm_us.sum()) - 1e3 * ms_per_step) / (2 * nl)

    # bf16 comparator (the vendor GEMM a user would otherwise call), timed both ways: inside a step of its own
    # over the same layer order with one event per launch (operands evicted like ours), and back to back
    bf16_us = bf16_b2b = None
    if not args.no_bf16:
        for l in layers:
            run_bf16(l)
        bf16_us = instrumented(layers, args.steps, [run_bf16])[0]
        bf16_b2b = [back_to_back(run_bf16, l, args.steps) for l in layers]
    quant_b2b = [back_to_back(run_quant, l, args.steps) for l in layers]
    gemm_b2b = [back_to_back(run_gemm, l, args.steps) for l in layers]

    per_layer = []
    for i, l in enumerate(layers):
        s = l["spec"]
        ops = 2.0 * s.macs
        act_bytes = 5.0 * s.M * s.K + 4.0 * s.M
        d = dict(name=s.name, M=s.M, K=s.K, N=s.N, K_o=l["w"].K_o,
                 gemm_us=round(float(gemm_us[i]), 2), quant_us=round(float(quant_us[i]), 2),
                 gemm_tops=round(ops / gemm_us[i] / 1e6, 1),
                 gemm_frac_peak=round(ops / gemm_us[i] / 1e6 / PEAK_INT8_TOPS, 4),
                 quant_gbs=round(act_bytes / quant_us[i] / 1e3, 1),
                 linear_us=round(float(linear_us[i]), 2),
                 gemm_back_to_back_us=round(gemm_b2b[i], 2), quant_back_to_back_us=round(quant_b2b[i], 2))
        if bf16_us is not None:
            d["bf16_us"] = round(float(bf16_us[i]), 2)
            d["bf16_back_to_back_us"] = round(bf16_b2b[i], 2)
            d["speedup_gemm_vs_bf16"] = round(float(bf16_us[i] / gemm_us[i]), 3)
            d["speedup_linear_vs_bf16"] = round(float(bf16_us[i] / linear_us[i]), 3)
            d["speedup_gemm_vs_bf16_back_to_back"] = round(bf16_b2b[i] / gemm_b2b[i], 3)
            d["speedup_linear_vs_bf16_back_to_back"] = round(bf16_b2b[i] / (gemm_b2b[i] + quant_b2b[i]), 3)
        per_layer.append(d)

    # ---- dominant kernel: the GEMM at the target shape (M=4680, 1536 -> 8960) ----------------
    tgt = [i for i, l in enumerate(layers) if (l["spec"].K, l["spec"].N) == (wl.HIDDEN, wl.FFN)]
    dom = tgt if tgt else [int(np.argmax(gemm_us))]
    dom_us = float(np.mean(gemm_us[dom]))
    s0 = layers[dom[0]]["spec"]
    dom_ops = 2.0 * s0.macs
    achieved = dom_ops / dom_us / 1e6
    # HBM-side bytes per launch come from committed rocprofv3 counter runs (bench.py cannot run the profiler)
    traffic_db = {}
    try:
        with open(os.path.join(ROOT, "profiles", "traffic_config2.json")) as fh:
            traffic_db = json.load(fh)
    except OSError:
        pass

    def traffic_of(kernel):
        t = traffic_db.get(kernel)
        return None if t is None else t["fetch_bytes"] + t["write_bytes"]

    traffic_note = ("not measured in this run: FETCH_SIZE + WRITE_SIZE of one dispatch from the committed counter run "
                    "profiles/traffic_config2.json (%s)" % traffic_db.get("provenance", "provenance not recorded"))
    dom_kernel = "qarvd_w8a8_dual_gemm M=%d K=%d N=%d" % (s0.M, s0.K, s0.N)
    dom_b2b = float(np.mean([gemm_b2b[i] for i in dom]))
    roofline = dict(bound="mfma", kernel=dom_kernel,
                    achieved=round(achieved, 1), peak=PEAK_INT8_TOPS, unit="TOP/s",
                    frac=round(achieved / PEAK_INT8_TOPS, 4), traffic=traffic_of(dom_kernel), traffic_source=traffic_note,
                    algorithmic_ops=dom_ops, avg_launch_us=round(dom_us, 2),
                    back_to_back_us=round(dom_b2b, 2),
                    frac_back_to_back=round(dom_ops / dom_b2b / 1e6 / PEAK_INT8_TOPS, 4))
    # the memory-bound kernel of the path
    qi = int(np.argmax(quant_us))
    sq = layers[qi]["spec"]
    q_kernel = "qarvd_quant_act M=%d K=%d" % (sq.M, sq.K)
    same = [i for i, l in enumerate(layers) if (l["spec"].M, l["spec"].K) == (sq.M, sq.K)]   # every launch of that shape
    q_us = float(np.mean([quant_us[i] for i in same]))
    q_bytes = 5.0 * sq.M * sq.K + 4.0 * sq.M
    quant_roof = dict(bound="hbm", kernel=q_kernel,
                      achieved=round(q_bytes / q_us / 1e3, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                      frac=round(q_bytes / q_us / 1e3 / PEAK_HBM_GBS, 4), traffic=traffic_of(q_kernel),
                      traffic_source=traffic_note,
                      algorithmic_bytes=q_bytes, avg_launch_us=round(q_us, 2), launches_averaged=len(same),
                      slowest_launch_us=per_layer[qi]["quant_us"])
    # quant_act, cold against warm, per activation shape: "cold" rotates over every input of that shape in the
    # workload (more than the 256 MB last-level cache in total), launches back to back with no events between;
    # "warm" repeats one launch on one input (served by the last-level cache); bf16 input beside fp32
    qa_protocol = []
    for (M_, K_) in sorted({(l["spec"].M, l["spec"].K) for l in layers}):
        group = [l for l in layers if (l["spec"].M, l["spec"].K) == (M_, K_)]
        in_bytes = sum(l["X"].numel() * 4 for l in group)
        bytes_ = 5.0 * M_ * K_ + 4.0 * M_
        cold = rotating(run_quant, group, max(2, args.steps // 4))
        warm = float(np.mean([quant_b2b[i] for i, l in enumerate(layers) if (l["spec"].M, l["spec"].K) == (M_, K_)]))
        entry = dict(M=M_, K=K_, inputs=len(group), input_bytes_total=in_bytes, cold_us=round(cold, 2), warm_us=round(warm, 2),
                     cold_gbs=round(bytes_ / cold / 1e3, 1), warm_gbs=round(bytes_ / warm / 1e3, 1),
                     cold_frac_hbm_peak=round(bytes_ / cold / 1e3 / PEAK_HBM_GBS, 4),
                     truly_cold=bool(in_bytes > (256 << 20)))
        if not args.no_bf16:
            def run_quant_bf16(l):
                q.quant_act(l["Xb"], l["perm"], l["w"].K_o, Xq=l["Xq"], s_x=l["sx"])
            cold_b = rotating(run_quant_bf16, group, max(2, args.steps // 4))
            entry["bf16_input_cold_us"] = round(cold_b, 2)
            entry["bf16_input_cold_gbs"] = round((3.0 * M_ * K_ + 4.0 * M_) / cold_b / 1e3, 1)
        qa_protocol.append(entry)

    out = dict(metric="INT8 TOPS of the dual-scale W8A8 linear (quant_act + dual GEMM); % of dense INT8 MFMA peak; "
                      "speedup vs bf16",
               value=round(value, 2), unit="TOPS", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=round(ms_per_step, 4), higher_is_better=True, scaling="weak", vs_baseline=None,
               dtype="int8", data="synthetic",
               config=dict(workload="config %d: %d DiT-block linears (M=%d tokens), quant_act + dual GEMM each"
                           % (args.config, nl, specs[0].M),
                           layers=nl, launches_per_step=2 * nl, out_dtype="bf16", gemm_variant=args.variant),
               frac_int8_peak=round(value / PEAK_INT8_TOPS, 4),
               event_overhead_us_per_launch=round(event_overhead_us, 2),
               roofline=roofline, quant_act_roofline=quant_roof, quant_act_cold_warm=qa_protocol)
    if bf16_us is not None:
        out["bf16_step_instrumented_ms"] = round(float(bf16_us.sum()) / 1e3, 4)   # the same layers as bf16 GEMMs, events included
        out["int8_step_instrumented_ms"] = round(float(quant_us.sum() + gemm_us.sum()) / 1e3, 4)
    if tgt:
        t = [per_layer[i] for i in tgt]

        def avg(key):
            return round(float(np.mean([x[key] for x in t])), 3)
        out["target_layer"] = dict(shape="M=4680 K=1536 N=8960",
                                   gemm_us=avg("gemm_us"), gemm_tops=avg("gemm_tops"), gemm_frac_peak=avg("gemm_frac_peak"),
                                   quant_us=avg("quant_us"), linear_us=avg("linear_us"),
                                   gemm_back_to_back_us=avg("gemm_back_to_back_us"),
                                   gemm_back_to_back_tops=round(float(np.mean([2.0 * layers[i]["spec"].macs / gemm_b2b[i] / 1e6
                                                                               for i in tgt])), 1),
                                   note="in-step figures: one event per launch (gemm_us, quant_us) or per layer (linear_us, "
                                        "bf16_us), operands evicted by the other layers; the bf16 comparator runs in a "
                                        "step of its own; back-to-back figures: one launch repeated on warm operands, "
                                        "both sides alike")
        if bf16_us is not None:
            for k in ("bf16_us", "bf16_back_to_back_us", "speedup_gemm_vs_bf16", "speedup_linear_vs_bf16",
                      "speedup_gemm_vs_bf16_back_to_back", "speedup_linear_vs_bf16_back_to_back"):
                out["target_layer"][k] = avg(k)
    try:
        issue_peak = q.probe_mfma_peak(20000)
        out["mfma_issue_peak"] = dict(tops=round(issue_peak, 1), frac_of_datasheet=round(issue_peak / PEAK_INT8_TOPS, 4),
                                      gemm_frac_of_issue_peak=round(achieved / issue_peak, 4),
                                      note="register-resident v_mfma_i32_32x32x32_i8 loop on every CU, measured in this run: "
                                           "what the MFMA pipes sustain on non-zero operands before the clock is pulled down")
    except Exception as e:  # diagnostic only
        out["mfma_issue_peak"] = dict(error=str(e))

    if not args.no_extras:
        side_measurements(out, args, layers, tgt, q, wl, torch, np, dev, run_quant, run_gemm)
    out["paper_context"] = "paper reports 1.30x end-to-end INT8 speedup and 1.97x size reduction on an NVIDIA A6000 " \
                           "with Triton kernels (whole pipeline, not this kernel)"

    # ---- CPU oracle on the host cores (reported baseline, bounded sample) -------------------
    if not args.no_cpu_baseline:
        import oracle
        # a bounded sample of the same workload: the layers with 16 or 64 planted outliers (two of the four
        # outlier settings of every shape; about 10 s of host time at full size)
        smp = [l for l in layers if l["spec"].n_outlier in (16, 64)] or layers[:1]
        cpu_ops, cpu_t = 0.0, 0.0
        for l in smp:
            s = l["spec"]
            Lh = wl.make_layer(s)
            qw = oracle.quantize_weight(Lh["W"])            # offline, untimed (as on the GPU side)
            t1 = time.perf_counter()
            Xq, sx = oracle.quant_act(Lh["X"], qw["perm"])
            oracle.dual_gemm(Xq, sx, qw["Wq"], qw["s_normal"], qw["s_outlier"], Lh["bias"], qw["K_o"],
                             want_acc=False, want_f32=False, want_bf16=True)
            cpu_t += time.perf_counter() - t1
            cpu_ops += 2.0 * s.macs
        # and on ONE host thread, the single config-1 layer (M=256, 1536 -> 1536)
        n_thr = oracle.num_threads()
        s1 = wl.config_layers(1)[0]
        L1 = wl.make_layer(s1)
        q1 = oracle.quantize_weight(L1["W"])
        oracle.set_num_threads(1)
        t1 = time.perf_counter()
        Xq1, sx1 = oracle.quant_act(L1["X"], q1["perm"])
        oracle.dual_gemm(Xq1, sx1, q1["Wq"], q1["s_normal"], q1["s_outlier"], L1["bias"], q1["K_o"],
                         want_acc=False, want_f32=False, want_bf16=True)
        one_t = time.perf_counter() - t1
        oracle.set_num_threads(n_thr)
        one_thread = dict(value=round(2.0 * s1.macs / one_t / 1e12, 5), unit="TOPS", cores=1, seconds=round(one_t, 3),
                          sample="config 1 (M=256, 1536 -> 1536), quant_act + dual_gemm")
        out["cpu_baseline"] = dict(value=round(cpu_ops / cpu_t / 1e12, 5), unit="TOPS", cores=oracle.num_threads(),
                                   kind="oracle", seconds=round(cpu_t, 2),
                                   sample="%d of the step's %d layers (q,k,v,o,ffn_up,ffn_down at M=%d with 16 and with 64 "
                                          "planted outliers), quant_act + dual_gemm, full size"
                                          % (len(smp), len(layers), smp[0]["spec"].M),
                                   one_thread=one_thread)
    out["layers"] = per_layer
    del layers
    torch.cuda.empty_cache()

    # ======================================================================= the other workloads, compact
    others = [int(c) for c in args.other_configs.split(",") if c.strip()] if not args.layers else []
    cfgs = []
    for cfg in others:
        if cfg == args.config:
            continue
        try:
            cfgs.append(compact_config(cfg, args, wl, torch, np, build_layers, timed_steps, instrumented, back_to_back,
                                       run_quant, run_gemm, run_bf16))
        except Exception as e:   # a workload that does not fit must not lose the headline
            cfgs.append(dict(config=cfg, error=repr(e)))
        torch.cuda.empty_cache()
    if cfgs:
        out["configs"] = cfgs
    print(json.dumps(out))


def compact_config(cfg, args, wl, torch, np, build_layers, timed_steps, instrumented, back_to_back,
                   run_quant, run_gemm, run_bf16):
    """One of the other workloads: whole-step value plus per-shape averages (in-step and back to back)."""
    specs = wl.config_layers(cfg)
    note = None
    if cfg == 3:
        # the 30 blocks repeat the same ten linears (outlier counts vary with depth): blocks 0, 14 and 29 are
        # timed and the step is those 30 layers; the stack of 300 takes ten times as long
        specs = [s for s in specs if s.tags.get("block") in (0, 14, 29)]
        note = "blocks 0, 14 and 29 of the 30-block stack (30 of its 300 layers); ms_per_step_full_stack = 10 x ms_per_step"
    layers = build_layers(specs, not args.no_bf16)
    steps = max(5, args.steps // 3)
    ms = timed_steps(layers, steps, 2)
    ops = sum(2.0 * l["spec"].macs for l in layers)
    quant_us, gemm_us = instrumented(layers, steps, [run_quant, run_gemm])

    def run_linear(l):
        run_quant(l)
        run_gemm(l)
    linear_us = instrumented(layers, steps, [run_linear])[0]       # one event per layer, like the bf16 step
    bf16_us = None
    if not args.no_bf16:
        for l in layers:
            run_bf16(l)
        bf16_us = instrumented(layers, steps, [run_bf16])[0]
    shapes = []
    for key in sorted({(l["spec"].M, l["spec"].K, l["spec"].N) for l in layers}):
        idx = [i for i, l in enumerate(layers) if (l["spec"].M, l["spec"].K, l["spec"].N) == key]
        M_, K_, N_ = key
        g = float(np.mean(gemm_us[idx]))
        qa = float(np.mean(quant_us[idx]))
        rep = layers[idx[len(idx) // 2]]
        lin = float(np.mean(linear_us[idx]))
        d = dict(M=M_, K=K_, N=N_, layers=len(idx), gemm_us=round(g, 2), quant_us=round(qa, 2), linear_us=round(lin, 2),
                 gemm_tops=round(2.0 * M_ * K_ * N_ / g / 1e6, 1),
                 gemm_frac_peak=round(2.0 * M_ * K_ * N_ / g / 1e6 / PEAK_INT8_TOPS, 4),
                 gemm_back_to_back_us=round(back_to_back(run_gemm, rep, steps), 2),
                 quant_back_to_back_us=round(back_to_back(run_quant, rep, steps), 2))
        if bf16_us is not None:
            b = float(np.mean(bf16_us[idx]))
            d["bf16_us"] = round(b, 2)
            d["bf16_back_to_back_us"] = round(back_to_back(run_bf16, rep, steps), 2)
            d["speedup_gemm_vs_bf16"] = round(b / g, 3)
            d["speedup_linear_vs_bf16"] = round(b / lin, 3)
        shapes.append(d)
    res = dict(config=cfg, layers=len(layers), steps=steps, ms_per_step=round(ms, 4),
               value=round(ops / (ms * 1e-3) / 1e12, 2), unit="TOPS",
               frac_int8_peak=round(ops / (ms * 1e-3) / 1e12 / PEAK_INT8_TOPS, 4), shapes=shapes)
    if note:
        res["note"] = note
        res["ms_per_step_full_stack"] = round(10.0 * ms, 3)
        # the paper's block has ten linears including the cross-attention output projection, the workload list of
        # the metric names nine: the stack without it, from the per-layer in-step times of the same pass
        cross_o = [i for i, l in enumerate(layers) if "cross_o" in l["spec"].name]
        if cross_o:
            t_all = float(linear_us.sum())
            t_wo = t_all - float(linear_us[cross_o].sum())
            ops_wo = ops - sum(2.0 * layers[i]["spec"].macs for i in cross_o)
            res["without_cross_attn_o"] = dict(layers=len(layers) - len(cross_o),
                                               ms_per_step_full_stack=round(10.0 * ms * t_wo / t_all, 3),
                                               value=round(ops_wo / (ms * 1e-3 * t_wo / t_all) / 1e12, 2),
                                               note="scaled from the step above by the share of the event-timed linears that remain")
    del layers
    return res


def side_measurements(out, args, layers, tgt, q, wl, torch, np, dev, run_quant, run_gemm):
    """Beside the headline (not part of `value`): the target layer with INT4 weights, W4A8 on the small-M shapes
    where the weights dominate the traffic, the chained FFN and the fused QKV layer."""
    def time_us(fn, reps=None):
        for _ in range(5):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps or args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / (reps or args.steps)

    if tgt:     # the same target layer with INT4 weights
        try:
            lt = layers[tgt[len(tgt) // 2]]
            w4 = q.quantize_weight(torch.from_numpy(wl.make_layer(lt["spec"])["W"]).to(dev), want_norms=False, bits=4)
            Xq4, sx4 = q.quant_act(lt["X"], w4.perm if w4.K_o else None, w4.K_o)
            us8 = time_us(lambda: run_gemm(lt))
            us4 = time_us(lambda: q.w8a8_dual_gemm(Xq4, sx4, w4, lt["bias"], lt["spec"].M, Y=lt["Y"]))
            us8 = min(us8, time_us(lambda: run_gemm(lt)))          # alternated, the better of two: the clock the chip
            us4 = min(us4, time_us(lambda: q.w8a8_dual_gemm(Xq4, sx4, w4, lt["bias"], lt["spec"].M, Y=lt["Y"])))   # holds drifts
            out["w4a8_target_layer"] = dict(layer=lt["spec"].name, gemm_us=round(us4, 2), w8a8_gemm_us=round(us8, 2),
                                            gemm_tops=round(2.0 * lt["spec"].macs / us4 / 1e6, 1),
                                            weight_bytes=int(w4.N * w4.kp // 2), int8_weight_bytes=int(w4.N * w4.kp),
                                            note="back-to-back launches of qarvd_w4a8_dual_gemm and of qarvd_w8a8_dual_gemm on "
                                                 "the target shape (compute-bound: halving the weight bytes cannot pay here, "
                                                 "and the INT4 path runs on the 64-byte-stage tiles only)")
            del w4, Xq4, sx4
        except Exception as e:  # diagnostic only
            out["w4a8_target_layer"] = dict(error=str(e))
    try:        # W4A8 where the weights are most of the bytes: the one-third-frame shapes of config 4 (M = 520)
        rows = []
        for name in ("cfg4.M520.ffn_up.c32", "cfg4.M520.ffn_down.c32", "cfg4.M520.attn.c32"):
            s = wl.find_layer(name)
            L = wl.make_layer(s)
            W = torch.from_numpy(L["W"]).to(dev)
            X = torch.from_numpy(L["X"]).to(dev)
            b = torch.from_numpy(L["bias"]).to(dev)
            w8 = q.quantize_weight(W, want_norms=False)
            w4 = q.quantize_weight(W, want_norms=False, bits=4)
            Xq, sx = q.quant_act(X, w8.perm if w8.K_o else None, w8.K_o)
            Y = torch.empty((s.M, s.N), dtype=torch.bfloat16, device=dev)
            us8 = time_us(lambda: q.w8a8_dual_gemm(Xq, sx, w8, b, s.M, Y=Y), 50)
            us4 = time_us(lambda: q.w8a8_dual_gemm(Xq, sx, w4, b, s.M, Y=Y), 50)
            rows.append(dict(layer=name, M=s.M, K=s.K, N=s.N, w8a8_gemm_us=round(us8, 2), w4a8_gemm_us=round(us4, 2),
                             int8_weight_bytes=int(w8.N * w8.kp), int4_weight_bytes=int(w4.N * w4.kp // 2)))
            del W, X, w8, w4, Xq
        out["w4a8_small_m"] = dict(rows=rows, note="back-to-back launches, M = 520 (one third of a latent frame): the shapes "
                                                   "where the weight matrix is most of the operand bytes")
    except Exception as e:  # diagnostic only
        out["w4a8_small_m"] = dict(error=str(e))
    if tgt and args.config == 2:   # FFN pair with the INT8 hand-over in the up-projection's epilogue
        try:
            up, down = wl.find_layer("cfg2.ffn_up.c16"), wl.find_layer("cfg2.ffn_down.c64")
            Lu, Ld = wl.make_layer(up), wl.make_layer(down)
            w2 = q.quantize_weight(torch.from_numpy(Ld["W"]).to(dev), want_norms=False)
            cmap = q.packed_channel_map(w2)
            W1 = torch.from_numpy(Lu["W"]).to(dev)
            W1p = torch.zeros((cmap.numel(), up.K), dtype=torch.float32, device=dev)
            b1p = torch.zeros(cmap.numel(), dtype=torch.float32, device=dev)
            W1p[cmap >= 0] = W1[cmap[cmap >= 0]]
            b1p[cmap >= 0] = torch.from_numpy(Lu["bias"]).to(dev)[cmap[cmap >= 0]]
            w1 = q.quantize_weight(W1p, want_norms=False)
            w1u = q.quantize_weight(W1, want_norms=False)
            b1, b2 = torch.from_numpy(Lu["bias"]).to(dev), torch.from_numpy(Ld["bias"]).to(dev)
            del W1, W1p
            M = up.M
            X = torch.from_numpy(Lu["X"]).to(dev).to(torch.bfloat16)
            Xq1 = torch.empty((M, q.packed_ld(w1.K, w1.K_o)), dtype=torch.int8, device=dev)
            sx1 = torch.empty(M, dtype=torch.float32, device=dev)
            H8 = torch.empty((M, q.packed_ld(w2.K, w2.K_o)), dtype=torch.int8, device=dev)
            Hb = torch.empty((M, up.N), dtype=torch.bfloat16, device=dev)
            sx2 = torch.empty(M, dtype=torch.float32, device=dev)
            Yf = torch.empty((M, down.N), dtype=torch.bfloat16, device=dev)
            s_mid = 0.03
            s_rows = torch.full((M,), s_mid, dtype=torch.float32, device=dev)

            def chained():
                q.quant_act(X, w1.perm if w1.K_o else None, w1.K_o, Xq=Xq1, s_x=sx1)
                q.w8a8_dual_gemm_q8(Xq1, sx1, w1, b1p, M, s_mid, q.ACT_GELU_TANH, Y8=H8)
                q.w8a8_dual_gemm(H8, s_rows, w2, b2, M, Y=Yf)

            def separate():
                q.quant_act(X, w1u.perm if w1u.K_o else None, w1u.K_o, Xq=Xq1, s_x=sx1)
                q.w8a8_dual_gemm(Xq1, sx1, w1u, b1, M, Y=Hb)
                g = torch.nn.functional.gelu(Hb, approximate="tanh")
                q.quant_act(g, w2.perm if w2.K_o else None, w2.K_o, Xq=H8, s_x=sx2)
                q.w8a8_dual_gemm(H8, sx2, w2, b2, M, Y=Yf)

            us_c, us_s = time_us(chained), time_us(separate)
            us_up8 = time_us(lambda: q.w8a8_dual_gemm_q8(Xq1, sx1, w1, b1p, M, s_mid, q.ACT_GELU_TANH, Y8=H8))
            us_upb = time_us(lambda: q.w8a8_dual_gemm(Xq1, sx1, w1u, b1, M, Y=Hb))
            ops = 2.0 * (up.macs + down.macs)
            out["chained_ffn"] = dict(shape="M=4680, 1536 -> 8960 -> 1536", chained_us=round(us_c, 1),
                                      separate_us=round(us_s, 1), speedup=round(us_s / us_c, 3),
                                      chained_tops=round(ops / us_c / 1e6, 1),
                                      up_gemm_int8_out_gelu_us=round(us_up8, 1), up_gemm_bf16_out_us=round(us_upb, 1),
                                      note="chained: quant_act, up GEMM with GELU + static INT8 hand-over in its epilogue "
                                           "(qarvd_w8a8_dual_gemm_q8), down GEMM; separate: quant_act, up GEMM to bf16, "
                                           "an elementwise GELU kernel (torch), quant_act, down GEMM")
            del w1, w1u, w2, X, Xq1, H8, Hb, Yf
        except Exception as e:  # diagnostic only
            out["chained_ffn"] = dict(error=str(e))
    if tgt and args.config == 2:   # q, k, v of one block as ONE layer (rows concatenated, one shared outlier set)
        try:
            names = ["cfg2.q.c16", "cfg2.k.c16", "cfg2.v.c16"]
            parts = [l for l in layers if l["spec"].name in names]
            Ws = [torch.from_numpy(wl.make_layer(l["spec"])["W"]).to(dev) for l in parts]
            wf = q.quantize_weight(torch.cat(Ws, 0), want_norms=False)
            bf = torch.cat([l["bias"] for l in parts])
            del Ws
            X0, M0 = parts[0]["X"], parts[0]["spec"].M
            Xqf = torch.empty((M0, q.packed_ld(wf.K, wf.K_o)), dtype=torch.int8, device=dev)
            sxf = torch.empty(M0, dtype=torch.float32, device=dev)
            Yf3 = torch.empty((M0, wf.N), dtype=torch.bfloat16, device=dev)

            def fused():
                q.quant_act(X0, wf.perm if wf.K_o else None, wf.K_o, Xq=Xqf, s_x=sxf)
                q.w8a8_dual_gemm(Xqf, sxf, wf, bf, M0, Y=Yf3)

            def three():
                for l in parts:
                    run_quant(l)
                    run_gemm(l)

            us_f, us_3 = time_us(fused), time_us(three)
            out["fused_qkv"] = dict(shape="M=4680, 1536 -> 3 x 1536 as one N=4608 layer", K_o=wf.K_o,
                                    fused_us=round(us_f, 1), separate_us=round(us_3, 1), speedup=round(us_3 / us_f, 3),
                                    note="one quant_act + one dual GEMM over the concatenated rows against three "
                                         "quant_act + GEMM pairs (which also read three different activations)")
            del wf, Xqf, Yf3
        except Exception as e:  # diagnostic only
            out["fused_qkv"] = dict(error=str(e))
    try:        # context: the vendor library's plain INT8 GEMM (INT32 out, no scales, no epilogue) on the same shapes
        rows = []
        for (M, K, N) in ((4680, 1536, 8960), (4680, 8960, 1536), (4680, 1536, 1536)):
            A = torch.randint(-127, 128, (M, K), dtype=torch.int8, device=dev)
            Bt = torch.randint(-127, 128, (N, K), dtype=torch.int8, device=dev).t()      # K x N, column-major
            us = time_us(lambda: torch._int_mm(A, Bt), 20)
            rows.append(dict(M=M, K=K, N=N, us=round(us, 1), tops=round(2.0 * M * N * K / us / 1e6, 1)))
            del A, Bt
        out["vendor_int8_gemm"] = dict(rows=rows, note="torch._int_mm (hipBLASLt INT8, INT32 output) launched back to back: "
                                                      "what the vendor's own kernels sustain on these shapes, for scale "
                                                      "beside gemm_back_to_back_us; not the same operation (no dual scale, "
                                                      "no de-quantization, four times the output bytes)")
    except Exception as e:  # diagnostic only
        out["vendor_int8_gemm"] = dict(error=str(e)[:200])


if __name__ == "__main__":
    main()
