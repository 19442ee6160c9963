"""Benchmark of the ASER per-layer calibration path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c1|c2|c4|c3.<layer>|c3]

One step = one pass of the whole hot path over one synthetic layer whose inputs already sit in
HBM: reset statistics, Gram accumulation (+ channel |x| sums), outlier selection / smoothing
diagonal, per-channel RTN and target T, Cholesky whitening, rank-r truncated SVD and L_A, L_B.
The default workload is the 4096 x 4096 Llama-7B-shaped projection (N = 32768 bf16 tokens, W4,
r = 64, f = 32).  `value` is the wall clock per layer over K such steps with sixteen layers in flight
(aser_calibrate_layers: Algorithm 1's loop over layers, one context and stream per layer in flight);
`one_layer_at_a_time_ms` and `stage_ms` are the same pass with a host wait after every layer.
Prints ONE JSON line.  The "roofline" object prices the dominant kernel (the
bf16 MFMA Gram update) by its algorithmic flops N n (n + 1); "cpu_baseline" times the CPU
oracle on a bounded sample on this host.  `--config c3` times the whole Llama-3-8B-shaped block
(seven layers on four input streams, plus the per-token A8 quantizer) and reports per-layer times.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HIP maps a process's streams onto four hardware queues unless told otherwise, and streams that share a queue
# run one after the other; sixteen queues let sixteen layers' chains really run side by side (more than that
# measured slower).  Read when the runtime initialises, so it is set before torch is imported.
if int(os.environ.get("GPU_MAX_HW_QUEUES", "0") or 0) < 16:
    os.environ["GPU_MAX_HW_QUEUES"] = "16"

METRIC = "per-layer ASER calibration ms + Gram/GEMM MFMA util %, 4096×4096 layer"
BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0
INT8_PEAK_TOPS = 5000.0
FP32_MFMA_PEAK_TFLOPS = 157.3
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gram_rtn_hbm_traffic.txt")


def measured_traffic():
    """HBM bytes per launch of the Gram and RTN kernels at workload c1, from the last line of
    profiles/gram_rtn_hbm_traffic.txt (written by `bench.py --traffic-summary` from two rocprofv3 --pmc
    runs of `bench.py --traffic-probe`, FETCH_SIZE and WRITE_SIZE, each scaled by a 1 GiB copy)."""
    try:
        with open(TRAFFIC_FILE) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch "):
                    return json.loads(line.split(" ", 1)[1])
    except OSError:
        pass
    return {}


def traffic_summary(fetch_dir, write_dir):
    """Reads the rocprofv3 result databases of the two counter runs and prints the summary that is kept
    as profiles/gram_rtn_hbm_traffic.txt."""
    import collections
    import glob
    import sqlite3
    agg = collections.defaultdict(list)
    for d in (fetch_dir, write_dir):
        dbs = sorted(glob.glob(os.path.join(d, "**", "*_results.db"), recursive=True))
        if not dbs:
            raise SystemExit("no *_results.db under %s" % d)
        con = sqlite3.connect(dbs[-1])
        for k, cn, v in con.execute("select kernel_name, counter_name, value from counters_collection"):
            agg[(k, cn)].append(float(v))
    copy = {cn: max(v) for (k, cn), v in agg.items() if "copyBuffer" in k or "CopyBuffer" in k}
    scale = {"FETCH_SIZE": (1 << 20) / copy["FETCH_SIZE"], "WRITE_SIZE": (1 << 20) / copy["WRITE_SIZE"]}
    print("HBM traffic of the Gram kernel and the RTN kernel, workload c1, MI355X: rocprofv3 --pmc FETCH_SIZE / "
          "WRITE_SIZE (KiB per dispatch).\n")
    print("Commands (from /tmp, TMPDIR=/tmp; one counter per run):")
    print("  rocprofv3 --pmc FETCH_SIZE -d gpurun_out/pmc_fetch -o fetch -- python3 bench.py --traffic-probe")
    print("  rocprofv3 --pmc WRITE_SIZE -d gpurun_out/pmc_write -o write -- python3 bench.py --traffic-probe")
    print("  python3 bench.py --traffic-summary gpurun_out/pmc_fetch gpurun_out/pmc_write > profiles/gram_rtn_hbm_traffic.txt")
    print("The probe runs a 1 GiB device-to-device copy (1 GiB read, 1 GiB written), the Gram kernel and the RTN "
          "kernel, three times each.\n")
    out = {}
    for (k, cn), v in sorted(agg.items()):
        if not any(t in k for t in ("gram_dma_kernel", "rtn_kernel", "opyBuffer")):
            continue
        print("%-90s %-11s launches=%d avg=%.6g KiB max=%.6g KiB" % (k[:90], cn, len(v), sum(v) / len(v), max(v)))
        for name in ("gram_dma_kernel", "rtn_kernel"):
            if name in k:
                out[name] = out.get(name, 0.0) + sum(v) / len(v) * 1024.0 * scale[cn]
    print("\nScale factors from the full-size copy (1048576 KiB read and written): FETCH_SIZE x%.3f, WRITE_SIZE x%.3f."
          % (scale["FETCH_SIZE"], scale["WRITE_SIZE"]))
    print("Bytes per launch = FETCH_SIZE x its factor + WRITE_SIZE x its factor:")
    print("traffic_bytes_per_launch " + json.dumps(out))


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(spec):
    """The CPU oracle as it stands, on the host cores.  A reduced layer (same statistics, same
    tokens/channel ratio) is timed first; every dominant stage is cubic in the size, so the full
    workload is predicted as t * (n / n_sample)^3.  If that prediction fits the budget the full
    workload itself is timed and reported; otherwise the scaled sample is."""
    import aser_synth as synth
    from oracle import aser_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))

    def run(sp):
        W = synth.make_weight(sp)
        X = synth.activations_as_f32(sp, synth.make_activations(sp))
        timings = {}
        t0 = time.perf_counter()
        orc.calibrate_layer(W, X, sp.bits, min(sp.f, sp.n), min(sp.r, sp.n, sp.m), timings=timings)
        return time.perf_counter() - t0, timings

    ns = 1536 if spec.n >= 1536 else spec.n
    sample = spec.with_(m=max(ns * spec.m // spec.n, 64), n=ns, tokens=int(ns * spec.tokens / spec.n))
    dt, timings = run(sample)
    scale = (spec.n / ns) ** 3
    if ns < spec.n and dt * scale <= 40.0:
        dt_full, timings = run(spec)
        return {"value": dt_full * 1e3, "unit": "ms", "cores": int(threads), "kind": "oracle",
                "sample": "the full workload: oracle.calibrate_layer on W %dx%d with %d tokens, %.1f s measured "
                          "(a %dx%d sample took %.2f s)" % (spec.m, spec.n, spec.tokens, dt_full, sample.m, sample.n, dt),
                "stages_s_measured": {k: round(v, 3) for k, v in timings.items()}}
    return {"value": dt * 1e3 * scale, "unit": "ms", "cores": int(threads), "kind": "oracle",
            "sample": "oracle.calibrate_layer on a %dx%d layer with %d tokens (same statistics), %.1f s measured, "
                      "scaled by (n/n_sample)^3 = %.2f" % (sample.m, sample.n, sample.tokens, dt, scale),
            "stages_s_measured": {k: round(v, 3) for k, v in timings.items()}}


def _gpu_present():
    import torch
    return torch.cuda.is_available()


def run_block(args):
    """--config c3: the Llama-3-8B-shaped block, layer by layer: one Gram per input stream (q, k, v share
    one, gate and up another), then smoothing, RTN, whitening, reconstruction and the per-token A8
    quantizer of the layer's smoothed input for each of the seven layers."""
    import torch
    import aser_synth as synth
    import paper_2411_07762_amd as aser

    dev = "cuda:0"
    torch.cuda.set_device(0)
    ctx = aser.Context(0)
    specs = [synth.CONFIGS[k] for k in synth.C3_LAYERS]
    streams, layers = {}, []
    for spec in specs:
        if spec.stream_id not in streams:
            log("generating stream %d: X %dx%d bf16" % (spec.stream_id, spec.tokens, spec.n))
            x_np = synth.make_activations(spec, workers=8)
            X = torch.from_numpy(x_np.view("int16")).to(dev).view(torch.bfloat16)
            del x_np
            streams[spec.stream_id] = {"X": X, "owner": None,
                                       "codes": torch.empty((spec.tokens, spec.n), dtype=torch.int8, device=dev),
                                       "scales": torch.empty(spec.tokens, dtype=torch.float32, device=dev)}
        st = streams[spec.stream_id]
        buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, packed=True)
        if st["owner"] is None:
            st["owner"] = buf
        else:                                    # layers of one input share its statistics
            buf.G, buf.abs_sum, buf.count = st["owner"].G, st["owner"].abs_sum, st["owner"].count
        W = torch.from_numpy(synth.make_weight(spec)).to(dev)
        layers.append((spec, st, buf, W))
        ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, spec.r))

    def block(ev=None):
        errs = []
        for i, (spec, st, buf, W) in enumerate(layers):
            if ev is not None:
                ev[i].record()
            first = st["owner"] is buf
            if first:
                buf.reset_statistics()
            aser.calibrate_layer(ctx, W, st["X"], buf, accumulate=first)
            ctx.check(aser.aser_quantize_act_rtn(ctx, st["X"], buf.mdiag, 8, st["codes"], st["scales"]))
            errs.append(buf.err)
        if ev is not None:
            ev[len(layers)].record()
        return errs

    for _ in range(args.warmup):
        block()
    torch.cuda.synchronize()
    layer_ms = [0.0] * len(layers)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(layers) + 1)]
        errs = block(ev)
        torch.cuda.synchronize()
        for i in range(len(layers)):
            layer_ms[i] += ev[i].elapsed_time(ev[i + 1]) / args.steps
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # The same block with four layers in flight (see block_in_flight), then the seven per-token quantizers spread
    # over the same streams.
    in_flight = None
    counts = [int(t) for t in args.in_flight.split(",") if t.strip()]
    if counts:
        pool = [torch.cuda.Stream(device=0) for _ in range(16)]
        s_, picked = aser.aser_pick_concurrent_streams([s.cuda_stream for s in pool], min(max(counts), len(layers)))
        ctx.check(s_)
        fctx = [aser.Context(0, stream=pool[i].cuda_stream) for i in picked]
        need = max(aser.aser_workspace_bytes(sp.m, sp.n, sp.r) for sp in specs)
        for c in fctx:
            c.ensure_workspace(need)
        order = sorted(range(len(layers)), key=lambda i: -(layers[i][0].m * layers[i][0].n * layers[i][0].n))
        owners = [(st, buf) for (_, st, buf, _) in layers if st["owner"] is buf]

        phase_ms = {"widest_gram_and_other_grams": 0.0, "layers": 0.0, "act_quant": 0.0}
        streams_f = [pool[i] for i in picked]
        layout4 = aser.ASER_CODES_INT4_PACKED

        def block_in_flight():
            # The widest layer has the longest chain by far (its Gram update is 23 of the block's 29 ms of Gram time,
            # its whitening and reconstruction 21 ms): its Gram update goes first and its five stages follow it on the
            # same stream, with no host wait in between.  The other Gram updates start when the wide one has ended
            # (two of them at a time fight for the device), on a second stream; the layers that need them wait for
            # that stream on the host and then run on the remaining contexts, next to the wide layer's chain.
            t_a = time.perf_counter()
            spec_w, st_w, buf_w, W_w = layers[order[0]]
            cA, sA = fctx[0], streams_f[0]
            with torch.cuda.stream(sA):
                buf_w.reset_statistics()
            cA.check(aser.aser_gram_accumulate(cA, st_w["X"], buf_w.G, buf_w.abs_sum, buf_w.count))
            gram_done = torch.cuda.Event()
            gram_done.record(sA)
            cA.check(aser.aser_smooth_outliers(cA, W_w, buf_w.abs_sum, buf_w.count, buf_w.f, buf_w.idx, buf_w.mdiag))
            cA.check(aser.aser_quantize_rtn(cA, W_w, buf_w.idx, buf_w.mdiag, buf_w.f, buf_w.bits, layout4, buf_w.codes,
                                            buf_w.scales, buf_w.T))
            s1, _ = aser.aser_whiten(cA, buf_w.G, buf_w.mdiag, 0.0, buf_w.S, want_info=False)
            cA.check(s1)
            cA.check(aser.aser_error_reconstruct_enqueue(cA, buf_w.T, buf_w.S, buf_w.r, buf_w.L_A, buf_w.L_B, buf_w.sigma,
                                                         idx=buf_w.idx, f=buf_w.f))
            cB, sB = fctx[1], streams_f[1]
            sB.wait_event(gram_done)
            for st, buf in owners:
                if buf is buf_w:
                    continue
                with torch.cuda.stream(sB):
                    buf.reset_statistics()
                cB.check(aser.aser_gram_accumulate(cB, st["X"], buf.G, buf.abs_sum, buf.count))
            sB.synchronize()
            t_b = time.perf_counter()
            rest = order[1:]
            descs = [aser.layer_desc(layers[i][3], layers[i][2]) for i in rest]
            s2 = aser.aser_calibrate_layers(fctx[1:], descs)
            if s2 != aser.ASER_OK:
                raise aser.AserError(s2, "aser_calibrate_layers on the block")
            s3, err_w, _ = aser.aser_finish(cA)
            cA.check(s3)
            t_c = time.perf_counter()
            for k, i in enumerate(order):
                spec, st, buf, _ = layers[i]
                c = fctx[k % len(fctx)]
                c.check(aser.aser_quantize_act_rtn(c, st["X"], buf.mdiag, 8, st["codes"], st["scales"]))
            torch.cuda.synchronize()
            t_d = time.perf_counter()
            for key, dt in (("widest_gram_and_other_grams", t_b - t_a), ("layers", t_c - t_b), ("act_quant", t_d - t_c)):
                phase_ms[key] += dt * 1e3 / args.steps
            out_e = {layers[i][0].name: d.err for i, d in zip(rest, descs)}
            out_e[spec_w.name] = err_w
            return out_e

        block_in_flight()
        torch.cuda.synchronize()
        phase_ms = dict.fromkeys(phase_ms, 0.0)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            errs_f = block_in_flight()
        in_flight = {"layers_in_flight": len(fctx), "block_ms": round((time.perf_counter() - t0) * 1e3 / args.steps, 3),
                     "phase_ms": {k: round(v, 3) for k, v in phase_ms.items()},
                     "whitened_error_max_rel_dev": max(abs(errs_f[sp.name] / e - 1.0) for (sp, _, _, _), e in zip(layers, errs))}
        log("block with %d layers in flight: %.2f ms" % (len(fctx), in_flight["block_ms"]))

        # The same block through ONE aser_calibrate_layers call: every layer a descriptor, the layers of one input
        # name the layer that accumulates its statistics (stats_from), widest layers first.
        by_name = {sp.name.split(".")[-1]: i for i, (sp, _, _, _) in enumerate(layers)}
        plan = [("down", None), ("gate", None), ("up", "gate"), ("q", None), ("k", "q"), ("v", "q"), ("o", None)]

        def block_one_call():
            pos, descs = {}, []
            for nm, src in plan:
                spec, st, buf, W = layers[by_name[nm]]
                pos[nm] = len(descs)
                if src is None:
                    descs.append(aser.layer_desc(W, buf, X=st["X"], clear_stats=True))
                else:
                    descs.append(aser.layer_desc(W, buf, stats_from=pos[src]))
            s_ = aser.aser_calibrate_layers(fctx, descs)
            if s_ != aser.ASER_OK:
                raise aser.AserError(s_, "aser_calibrate_layers on the whole block")
            for k, (nm, _) in enumerate(plan):
                spec, st, buf, _ = layers[by_name[nm]]
                c = fctx[k % len(fctx)]
                c.check(aser.aser_quantize_act_rtn(c, st["X"], buf.mdiag, 8, st["codes"], st["scales"]))
            torch.cuda.synchronize()
            return {layers[by_name[nm]][0].name: d.err for (nm, _), d in zip(plan, descs)}

        if all(nm in by_name for nm, _ in plan):
            block_one_call()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                errs_o = block_one_call()
            in_flight["block_ms_through_one_call"] = round((time.perf_counter() - t0) * 1e3 / args.steps, 3)
            in_flight["whitened_error_max_rel_dev_one_call"] = max(abs(errs_o[sp.name] / e - 1.0) for (sp, _, _, _), e in zip(layers, errs))
            log("block through one aser_calibrate_layers call: %.2f ms" % in_flight["block_ms_through_one_call"])
        for c in fctx:
            c.close()

    # W4A8 layer-output error of every layer (Sec. 5.3 error figure metric, relative to ||X W^T||_F) on a sample of
    # its calibration tokens: with the factors, and for RTN alone
    sample = 2048
    w4a8 = {}
    for spec, st, buf, W in layers:
        ctx.ensure_workspace(aser.aser_output_error_workspace_bytes(spec.m, spec.n, sample, spec.r))
        vals = {}
        for comp in (True, False):
            s_, e, yn = aser.aser_layer_output_error(ctx, W, st["X"][:sample], buf.mdiag, buf.codes, aser.ASER_CODES_INT4_PACKED,
                                                     buf.scales, buf.L_A if comp else None, buf.L_B if comp else None,
                                                     spec.r if comp else 0, 8)
            ctx.check(s_)
            vals["compensated" if comp else "rtn_only"] = e / yn
        w4a8[spec.name] = vals
    for spec, st, buf, W in layers:
        ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, spec.r))

    # the Gram kernel of the widest stream alone, for the roofline object
    spec, st, buf, _ = layers[-1]
    G2 = torch.zeros_like(buf.G)
    ctx.check(aser.aser_gram_accumulate(ctx, st["X"], G2))
    torch.cuda.synchronize()
    reps = max(3, args.steps)
    pairs = []
    for _ in range(reps):                       # one event pair per launch, the block between two launches
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ctx.check(aser.aser_gram_accumulate(ctx, st["X"], G2))
        e1.record()
        pairs.append((e0, e1))
        block()
    torch.cuda.synchronize()
    gram_ms = sum(a.elapsed_time(b) for a, b in pairs) / reps
    gram_flops = float(spec.tokens) * spec.n * (spec.n + 1)
    gram_tflops = gram_flops / (gram_ms * 1e-3) / 1e12
    out = {
        "metric": "ASER calibration ms, Llama-3-8B-shaped block (7 layers, 4 Grams, W4A8)", "value": wall_ms, "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall_ms, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "c3: q 4096x4096, k/v 1024x4096, o 4096x4096, gate/up 14336x4096, down 4096x14336; "
                               "131072 bf16 tokens per input stream; W4 per-channel RTN, A8 per-token, r=64, f=32"},
        "layer_ms": {sp.name: round(ms, 3) for (sp, _, _, _), ms in zip(layers, layer_ms)},
        "block_with_layers_in_flight": in_flight,
        "whitened_error": {sp.name: e for (sp, _, _, _), e in zip(layers, errs)},
        "w4a8_output_error_relative": {"sample_tokens": sample, "layers": w4a8},
        "roofline": {"kernel": "gram_dma_kernel (Gram update of the 14336-channel stream)", "bound": "mfma",
                     "achieved": gram_tflops, "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gram_tflops / BF16_PEAK_TFLOPS, "traffic": None,
                     "algorithmic_flops_per_launch": gram_flops, "avg_launch_ms": gram_ms},
    }
    log("layer ms:", out["layer_ms"], "block %.2f ms" % wall_ms)
    print(json.dumps(out))


def trace_summary(result_dir, note):
    """Prints the per-kernel totals of a rocprofv3 --kernel-trace --stats run (kept under profiles/): first the
    launches on the default stream (the one-layer-at-a-time pass and the kernel timing loops: kernels that have
    the device to themselves, which is what the roofline figures refer to), then the launches on the other
    streams (the layers in flight, whose kernels share the device and take longer each)."""
    import collections
    import glob
    import sqlite3
    dbs = sorted(glob.glob(os.path.join(result_dir, "**", "*_results.db"), recursive=True))
    if not dbs:
        raise SystemExit("no *_results.db under %s" % result_dir)
    con = sqlite3.connect(dbs[-1])
    agg = {True: collections.defaultdict(list), False: collections.defaultdict(list)}
    for name, stream, dur in con.execute("select name, stream, duration from kernels"):
        agg[stream is None or "Default" in stream][name].append(dur * 1e-3)
    print(note)
    for alone, title in ((True, "Launches on the default stream (kernels running alone)"),
                         (False, "Launches on the streams of the layers in flight")):
        rows = sorted(agg[alone].items(), key=lambda kv: -sum(kv[1]))[:40]
        if not rows:
            continue
        total = sum(sum(v) for v in agg[alone].values())
        print("\n%s; durations in microseconds:" % title)
        print("%-96s %6s %12s %10s %6s" % ("kernel", "calls", "total_us", "avg_us", "pct"))
        for name, v in rows:
            print("%-96s %6d %12.1f %10.2f %6.2f" % (name[:96], len(v), sum(v), sum(v) / len(v), 100.0 * sum(v) / total))


def clock_summary(result_dir, note):
    """Prints, per MFMA-bound kernel of a `rocprofv3 --kernel-trace --pmc GRBM_GUI_ACTIVE` run, the average
    duration and the shader clock it ran at: GRBM_GUI_ACTIVE counts the cycles a die (XCD) is busy and the tool
    sums it over the 8 dies, so cycles / 8 / duration is the clock (kept under profiles/)."""
    import collections
    import glob
    import sqlite3
    dbs = sorted(glob.glob(os.path.join(result_dir, "**", "*_results.db"), recursive=True))
    if not dbs:
        raise SystemExit("no *_results.db under %s" % result_dir)
    con = sqlite3.connect(dbs[-1])
    dur = {r[0]: r[2] - r[1] for r in con.execute("select dispatch_id, start, end from kernels")}
    agg = collections.OrderedDict()
    for did, name, cn, v in con.execute("select dispatch_id, kernel_name, counter_name, value from counters_collection"):
        if cn != "GRBM_GUI_ACTIVE" or did not in dur:
            continue
        e = agg.setdefault(did, [name, 0.0])
        e[1] += v
    per = collections.OrderedDict()
    for did, (name, cyc) in agg.items():
        if dur[did] < 100e3:                      # launches under 100 us: the counter's start and stop weigh too much
            continue
        per.setdefault(name, []).append((dur[did] * 1e-3, cyc / 8.0 / dur[did]))
    print(note)
    print("\nKernels of at least 100 us (clock = GRBM_GUI_ACTIVE / 8 / duration):")
    print("%-100s %5s %10s %9s %9s %9s" % ("kernel", "calls", "avg_us", "GHz_avg", "GHz_min", "GHz_max"))
    for name, v in sorted(per.items(), key=lambda kv: -sum(x[0] for x in kv[1])):
        ghz = [x[1] for x in v]
        print("%-100s %5d %10.1f %9.2f %9.2f %9.2f" % (name[:100], len(v), sum(x[0] for x in v) / len(v),
                                                      sum(ghz) / len(ghz), min(ghz), max(ghz)))


def extras(ctx, aser, torch, spec, buf, W, X, reps):
    """Timings of the rows beyond the calibration path, on the layer the step has just calibrated: the full
    spectrum with the rank rule of Eq. 9 and the effective rank of Eq. 3-4, the W4A8 layer-output error on a
    token sample, and the compensated inference kernel (int8 MFMA) with and without its rank-r branch."""
    dev = X.device
    res = {}

    def timed(fn, n=3):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # full spectrum of T S, rank from alpha, effective rank
    k = min(spec.m, spec.n)
    ctx.ensure_workspace(aser.aser_spectrum_workspace_bytes(spec.m, spec.n, True))
    sig = torch.empty(k, dtype=torch.float64, device=dev)
    ms = timed(lambda: ctx.check(aser.aser_singular_values(ctx, buf.T, buf.S, sig)), 2)
    ranks = {}
    for alpha in (0.1, 0.075, 0.05, 0.03, 0.015):
        st, r_sel, _ = aser.aser_select_rank(ctx, sig, alpha)
        ctx.check(st)
        ranks[str(alpha)] = r_sel
    st, erank = aser.aser_effective_rank(ctx, sig)
    ctx.check(st)
    pass_bytes = 16.0 * k ** 3 / 3.0
    res["spectrum"] = {"ms": ms, "k": k, "rank_from_alpha": ranks, "effective_rank_of_T_S": erank,
                       "tridiagonalisation_algorithmic_bytes": pass_bytes,
                       "note": "bound by the passes over the fp64 trailing matrix (16 k^3 / 3 bytes, served by the "
                               "last-level cache when the matrix fits) and by 2 (k - 2) launches"}
    # a rank beyond the widest subspace block of the iteration (the rule of Eq. 9 can ask for one): the dense fp64 solver
    r_big = 200
    if min(spec.m, spec.n) >= r_big and min(spec.m, spec.n) <= 16384 and spec.r <= 128:
        ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, r_big))
        la = torch.empty((spec.m, r_big), dtype=torch.float32, device=dev)
        lb = torch.empty((r_big, spec.n), dtype=torch.float32, device=dev)
        sg = torch.empty(r_big, dtype=torch.float32, device=dev)
        errs = []

        def big():
            st_, e_, _ = aser.aser_error_reconstruct(ctx, buf.T, buf.S, r_big, la, lb, sg)
            ctx.check(st_)
            errs.append(e_)

        res["reconstruct_rank_200_dense_solver"] = {"ms": timed(big, 1), "whitened_error": errs[-1]}
        del la, lb, sg
    # the two passes around a caller's own weight quantizer (closing remark of Sec. 4.1): W_s out, T = W M - W_q in;
    # buffers rotate so that a weight smaller than the last-level cache is still read from HBM
    mn = spec.m * spec.n
    nrot = 4 if mn * 4 < (256 << 20) else 1
    w_in = [W] + [W.clone() for _ in range(nrot - 1)]
    w_s = [torch.empty_like(W) for _ in range(nrot)]
    t_out = [torch.empty_like(W) for _ in range(nrot)]
    turn = [0]

    def pass_ws():
        i = turn[0] = (turn[0] + 1) % nrot
        ctx.check(aser.aser_smoothed_weight(ctx, w_in[i], buf.idx, spec.f, w_s[i]))

    def pass_t():
        i = turn[0] = (turn[0] + 1) % nrot
        ctx.check(aser.aser_quant_target(ctx, w_in[i], buf.mdiag, w_s[i], t_out[i]))

    for _ in range(nrot):
        pass_ws()
    ms_ws, ms_t = timed(pass_ws, 4 * nrot), timed(pass_t, 4 * nrot)
    res["passes_around_another_weight_quantizer"] = {
        "smoothed_weight_us": ms_ws * 1e3, "smoothed_weight_gbs": 8.0 * mn / (ms_ws * 1e6),
        "quant_target_us": ms_t * 1e3, "quant_target_gbs": 12.0 * mn / (ms_t * 1e6),
        "algorithmic_bytes": "8 m n and 12 m n (fp32 W in, W_s out; W and W_q in, T out)"}
    del w_in, w_s, t_out
    # layer-output error, W4A8 and W4A6, compensated and not, on a sample of the calibration tokens
    sample = min(2048, spec.tokens)
    ctx.ensure_workspace(aser.aser_output_error_workspace_bytes(spec.m, spec.n, sample, spec.r))
    layout = aser.ASER_CODES_INT4_PACKED if buf.packed else aser.ASER_CODES_INT8
    oe = {}
    for act_bits, comp in ((8, True), (8, False), (6, True), (6, False)):
        st, e, yn = aser.aser_layer_output_error(ctx, W, X[:sample], buf.mdiag, buf.codes, layout, buf.scales,
                                                 buf.L_A if comp else None, buf.L_B if comp else None,
                                                 spec.r if comp else 0, act_bits)
        ctx.check(st)
        oe["W%dA%d_%s" % (spec.bits, act_bits, "compensated" if comp else "rtn_only")] = e / yn
    ms = timed(lambda: aser.aser_layer_output_error(ctx, W, X[:sample], buf.mdiag, buf.codes, layout, buf.scales,
                                                    buf.L_A, buf.L_B, spec.r, 8), 3)
    # the W8 variants of Sec. 5.1 (A8, A6, A4) on the same layer, calibrated once more with 8-bit weights
    if spec.bits != 8 and spec.m * spec.n <= (1 << 26):
        buf8 = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, 8, packed=False)
        aser.calibrate_layer(ctx, W, X, buf8)
        ctx.ensure_workspace(aser.aser_output_error_workspace_bytes(spec.m, spec.n, sample, spec.r))
        for act_bits in (8, 6, 4):
            for comp in (True, False):
                st, e, yn = aser.aser_layer_output_error(ctx, W, X[:sample], buf8.mdiag, buf8.codes, aser.ASER_CODES_INT8,
                                                         buf8.scales, buf8.L_A if comp else None, buf8.L_B if comp else None,
                                                         spec.r if comp else 0, act_bits)
                ctx.check(st)
                oe["W8A%d_%s" % (act_bits, "compensated" if comp else "rtn_only")] = e / yn
        del buf8
    res["layer_output_error"] = {"ms": ms, "sample_tokens": sample, "relative_to_exact_output_norm": oe}
    # compensated inference kernel on the whole calibration stream (tokens x n int8 codes)
    if spec.n % 32 == 0:
        xq = torch.empty((spec.tokens, spec.n), dtype=torch.int8, device=dev)
        xs = torch.empty(spec.tokens, dtype=torch.float32, device=dev)
        ctx.check(aser.aser_quantize_act_rtn(ctx, X, buf.mdiag, 8, xq, xs))
        Y = torch.empty((spec.tokens, spec.m), dtype=torch.float32, device=dev)
        ctx.ensure_workspace(aser.aser_forward_workspace_bytes(spec.tokens, spec.n, spec.m, spec.r))
        fw = {}
        for name, r_use, split in (("no_compensation", 0, False), ("rank_r_bf16", spec.r, False), ("rank_r_split", spec.r, True)):
            fw[name] = timed(lambda: ctx.check(aser.aser_compensated_forward(
                ctx, xq, xs, buf.codes, layout, buf.scales, buf.L_A if r_use else None, buf.L_B if r_use else None,
                r_use, split, Y)), max(3, reps // 2))
        ops = 2.0 * spec.tokens * spec.n * spec.m
        res["compensated_forward"] = {
            "ms": fw, "tokens": spec.tokens,
            "roofline": {"kernel": "cf_dma_kernel (int8 MFMA, 256 x 256 tiles, LDS-direct loads, int4 weight codes widened after the LDS read)",
                         "bound": "mfma",
                         "achieved": ops / (fw["no_compensation"] * 1e-3) / 1e12, "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                         "frac": ops / (fw["no_compensation"] * 1e-3) / 1e12 / INT8_PEAK_TOPS},
            "overhead_of_rank_r_branch": {"measured_bf16": fw["rank_r_bf16"] / fw["no_compensation"] - 1.0,
                                          "measured_split": fw["rank_r_split"] / fw["no_compensation"] - 1.0,
                                          "paper_flops_ratio_2r_over_d": 2.0 * spec.r / spec.n}}
        # Context, not a target and not part of the path: the vendor library's plain GEMMs of the same shapes
        # through torch (no scales, no rank-r branch, int32 output for int8; the full X^T X, of which the Gram
        # kernel computes the lower-triangle tiles).
        lib = {}
        try:
            if X.dtype == torch.bfloat16:
                ms_l = timed(lambda: torch.matmul(X.t(), X), 3)
                lib["bf16_full_XtX"] = {"ms": ms_l, "tflops": 2.0 * spec.tokens * spec.n * spec.n / (ms_l * 1e-3) / 1e12}
            wq8 = torch.randint(-127, 128, (spec.m, spec.n), dtype=torch.int8, device=dev)
            ms_l = timed(lambda: torch._int_mm(xq, wq8.t()), 3)
            lib["int8_x_wT_int32_out"] = {"ms": ms_l, "tops": ops / (ms_l * 1e-3) / 1e12}
            del wq8
        except Exception as exc:                          # an op the installed torch build lacks: report, do not fail
            lib["unavailable"] = repr(exc)[:200]
        res["library_gemm_same_shapes"] = lib
        del xq, Y
    return res


def layers_in_flight(aser, torch, spec, X, Ws, n_ctx, n_layers, warmup):
    """Throughput of Algorithm 1's loop over layers with n_ctx layers in flight (aser_calibrate_layers: one host
    thread, n_ctx contexts with their own streams, buffers and workspaces; every layer is a full pass of the
    workload from the shared X, statistics cleared first).  Returns wall-clock ms per layer and the errors."""
    # streams that really run side by side: the runtime maps streams to four hardware queues per process
    pool = [torch.cuda.Stream(device=0) for _ in range(max(16, 4 * n_ctx))]
    st, picked = aser.aser_pick_concurrent_streams([s.cuda_stream for s in pool], n_ctx)
    if st != aser.ASER_OK:
        raise aser.AserError(st, "aser_pick_concurrent_streams")
    streams = [pool[i] for i in picked]
    n_ctx = len(streams)
    ctxs = [aser.Context(0, stream=s.cuda_stream) for s in streams]
    # per layer: its outputs; G, T and S are intermediates of the context that gets the layer
    outs = [aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, packed=True, intermediates=False)
            for _ in range(n_layers)]
    need = aser.aser_layer_workspace_bytes(aser.layer_desc(Ws[0], outs[0], X=X))
    for c in ctxs:
        c.ensure_workspace(need)
    torch.cuda.synchronize()

    def run(count):
        descs = [aser.layer_desc(Ws[k % len(Ws)], outs[k], X=X) for k in range(count)]
        st = aser.aser_calibrate_layers(ctxs, descs)
        if st != aser.ASER_OK:
            bad = next(k for k, d in enumerate(descs) if d.status != aser.ASER_OK)
            raise aser.AserError(st, "layer %d of %d in flight: status %d" % (bad, n_ctx, descs[bad].status))
        return [d.err for d in descs]

    run(min(max(warmup, n_ctx), n_layers))                # untimed
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    errs = run(n_layers)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for c in ctxs:
        c.close()
    return wall * 1e3 / n_layers, errs, n_ctx


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="c1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="run only a 1 GiB copy, the Gram kernel and the RTN kernel (for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--traffic-summary", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="print the summary of the two counter runs (no GPU needed)")
    ap.add_argument("--trace-summary", nargs=2, metavar=("RESULT_DIR", "NOTE"),
                    help="print the per-kernel totals of a rocprofv3 --kernel-trace --stats run (no GPU needed)")
    ap.add_argument("--clock-summary", nargs=2, metavar=("RESULT_DIR", "NOTE"),
                    help="print per-kernel shader clocks of a rocprofv3 --kernel-trace --pmc GRBM_GUI_ACTIVE run (no GPU needed)")
    ap.add_argument("--no-extras", action="store_true", help="skip the timings of the rows beyond the calibration path")
    ap.add_argument("--in-flight", default="16,4,2", help="layers in flight (aser_calibrate_layers): the first count is the "
                    "headline's, the others are reported beside it; 1 or empty: one layer at a time is the headline")
    args = ap.parse_args()
    if args.traffic_summary:
        return traffic_summary(*args.traffic_summary)
    if args.trace_summary:
        return trace_summary(*args.trace_summary)
    if args.clock_summary:
        return clock_summary(*args.clock_summary)
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    if args.config == "c3":
        if not _gpu_present():
            print("bench.py needs a GPU", file=sys.stderr)
            sys.exit(2)
        return run_block(args)

    import numpy as np
    import torch
    import aser_synth as synth
    import paper_2411_07762_amd as aser

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    spec = synth.CONFIGS[args.config]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    log("generating %s: W %dx%d, X %dx%d %s" % (spec.name, spec.m, spec.n, spec.tokens, spec.n, spec.x_dtype))
    W_np = synth.make_weight(spec)
    n_rot = 4                                   # rotate weight buffers so the 256 MB cache does not flatter RTN
    Ws = [torch.from_numpy(W_np).to(dev) for _ in range(n_rot)]
    x_np = synth.make_activations(spec, workers=8)
    if spec.x_dtype == "bf16":
        X = torch.from_numpy(x_np.view(np.int16)).to(dev).view(torch.bfloat16)
    else:
        X = torch.from_numpy(x_np).to(dev)
    del x_np

    ctx = aser.Context(0)
    buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, packed=True)
    ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, spec.r))
    layout = aser.ASER_CODES_INT4_PACKED
    stage_names = ["reset", "gram", "smooth", "rtn", "whiten", "reconstruct"]

    def step(i, ev=None):
        W = Ws[i % n_rot]

        def mark(k):
            if ev is not None:
                ev[k].record()

        mark(0)
        buf.reset_statistics()
        mark(1)
        ctx.check(aser.aser_gram_accumulate(ctx, X, buf.G, buf.abs_sum, buf.count))
        mark(2)
        ctx.check(aser.aser_smooth_outliers(ctx, W, buf.abs_sum, buf.count, buf.f, buf.idx, buf.mdiag))
        mark(3)
        ctx.check(aser.aser_quantize_rtn(ctx, W, buf.idx, buf.mdiag, buf.f, buf.bits, layout, buf.codes, buf.scales, buf.T))
        mark(4)
        st, info = aser.aser_whiten(ctx, buf.G, buf.mdiag, 0.0, buf.S, want_info=False)   # pivot check at the layer's one sync
        ctx.check(st)
        mark(5)
        st, err, _ = aser.aser_error_reconstruct(ctx, buf.T, buf.S, buf.r, buf.L_A, buf.L_B, buf.sigma, idx=buf.idx, f=buf.f)
        ctx.check(st)
        mark(6)
        return err

    if args.traffic_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        step(0)
        for _ in range(3):
            dst.copy_(src)                       # plain copy of known size: 1 GiB read, 1 GiB written
            ctx.check(aser.aser_gram_accumulate(ctx, X, buf.G))
            ctx.check(aser.aser_quantize_rtn(ctx, Ws[0], buf.idx, buf.mdiag, buf.f, buf.bits, layout, buf.codes,
                                             buf.scales, buf.T))
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30}))
        return

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    stage_ms = [0.0] * len(stage_names)
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(7)]
        err = step(i, ev)
        torch.cuda.synchronize()
        for k in range(6):
            stage_ms[k] += ev[k].elapsed_time(ev[k + 1])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = [s / args.steps for s in stage_ms]

    # The headline: args.steps layers through aser_calibrate_layers with the first count of --in-flight layers in
    # flight (contexts and streams of their own), wall clock over all of them.  The one-layer-at-a-time figure
    # above stays in the line next to it, with its stage times.
    in_flight = {}
    counts = [int(t) for t in args.in_flight.split(",") if t.strip() and int(t) > 1]
    head_n, head_ms, head_layers = 1, ms_per_step, args.steps
    for nl in counts:
        try:
            # whole rounds of nl layers (at least `steps`): a last round with fewer layers in flight than the
            # others would time a different configuration
            timed_layers = -(-max(args.steps, nl) // nl) * nl
            ms_l, errs_l, got = layers_in_flight(aser, torch, spec, X, Ws, nl, timed_layers, args.warmup)
        except Exception as exc:                          # the one-at-a-time figure then stays the headline; say why
            log("layers in flight %d failed: %r" % (nl, exc))
            in_flight[str(nl)] = {"failed": repr(exc)[:200]}
            continue
        in_flight[str(nl)] = {"ms_per_layer": round(ms_l, 4), "layers_per_s": round(1e3 / ms_l, 2),
                              "concurrent_streams": got, "layers_timed": timed_layers,
                              "whitened_error_max_rel_dev": max(abs(e / err - 1.0) for e in errs_l)}
        log("layers in flight %d (on %d concurrent streams): %.3f ms per layer" % (nl, got, ms_l))
        if nl == counts[0]:
            head_n, head_ms, head_layers = got, in_flight[str(nl)]["ms_per_layer"], timed_layers

    # Dominant kernel alone: the Gram MFMA kernel (no statistics pass), HIP events on the launch stream, one
    # pair around every launch, and a whole layer step between two launches as in the pipeline.  (Launched
    # back to back the kernel heats the chip and the clock drops within milliseconds: ten such launches
    # climb from 490 to 590 us at c1, a rate no calibration run sees.)
    reps = max(10, args.steps)
    G2 = torch.zeros_like(buf.G)
    ctx.check(aser.aser_gram_accumulate(ctx, X, G2))
    torch.cuda.synchronize()
    pairs = []
    for i in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        # a streaming kernel in front, as the statistics pass is in the pipeline: the step before ended with
        # a host synchronisation, and the Gram launch is not meant to start on an idle device
        ctx.check(aser.aser_quantize_rtn(ctx, Ws[i % n_rot], buf.idx, buf.mdiag, buf.f, buf.bits, layout, buf.codes,
                                         buf.scales, buf.T))
        e0.record()
        ctx.check(aser.aser_gram_accumulate(ctx, X, G2))
        e1.record()
        step(i)
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    gram_ms = sum(a.elapsed_time(b) for a, b in pairs) / reps
    e0, e1 = pairs[0]
    gram_flops = float(spec.tokens) * spec.n * (spec.n + 1)
    gram_tflops = gram_flops / (gram_ms * 1e-3) / 1e12

    # Bandwidth kernel: RTN + target (algorithmic bytes 8.5 m n + 4 m), rotating weight buffers.
    for i in range(4):                           # untimed: the first launches after another kernel run slower
        ctx.check(aser.aser_quantize_rtn(ctx, Ws[i % n_rot], buf.idx, buf.mdiag, buf.f, buf.bits, layout, buf.codes,
                                         buf.scales, buf.T))
    e0.record()
    for i in range(reps):
        ctx.check(aser.aser_quantize_rtn(ctx, Ws[i % n_rot], buf.idx, buf.mdiag, buf.f, buf.bits, layout, buf.codes,
                                         buf.scales, buf.T))
    e1.record()
    torch.cuda.synchronize()
    rtn_ms = e0.elapsed_time(e1) / reps
    rtn_bytes = 8.5 * spec.m * spec.n + 4.0 * spec.m
    rtn_gbs = rtn_bytes / (rtn_ms * 1e-3) / 1e9

    # Per-token activation quantizer (a7) on the calibration stream: algorithmic bytes 3 N n + 4 N for bf16 X.
    act_codes = torch.empty((spec.tokens, spec.n), dtype=torch.int8, device=dev)
    act_scales = torch.empty(spec.tokens, dtype=torch.float32, device=dev)
    ctx.check(aser.aser_quantize_act_rtn(ctx, X, buf.mdiag, 8, act_codes, act_scales))
    e0.record()
    for i in range(reps):
        ctx.check(aser.aser_quantize_act_rtn(ctx, X, buf.mdiag, 8, act_codes, act_scales))
    e1.record()
    torch.cuda.synchronize()
    act_ms = e0.elapsed_time(e1) / reps
    act_bytes = (X.element_size() + 1.0) * spec.tokens * spec.n + 4.0 * spec.tokens
    act_gbs = act_bytes / (act_ms * 1e-3) / 1e9
    del act_codes

    # Context for the two bandwidth kernels: what a plain device-to-device copy that moves the same number of bytes
    # (half read, half written) reaches on this device, over buffers that rotate beyond the 256 MB cache.
    def plain_copy_gbs(total_bytes):
        half = int(total_bytes) // 2 // 4 * 4
        nbuf = max(2, int((600 << 20) // max(half, 1)) + 1)
        srcs = [torch.empty(half, dtype=torch.uint8, device=dev) for _ in range(nbuf)]
        dsts = [torch.empty(half, dtype=torch.uint8, device=dev) for _ in range(nbuf)]
        for i in range(4):
            dsts[i % nbuf].copy_(srcs[i % nbuf])
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for i in range(reps):
            dsts[i % nbuf].copy_(srcs[i % nbuf])
        c1.record()
        torch.cuda.synchronize()
        return 2.0 * half / (c0.elapsed_time(c1) / reps * 1e-3) / 1e9

    copy_rtn_gbs = plain_copy_gbs(rtn_bytes)
    copy_act_gbs = plain_copy_gbs(act_bytes)

    # What a loop of nothing but MFMA instructions reaches on this device (the clock drops under that load):
    # one workgroup of four wavefronts per compute unit, which is the occupancy of the Gram kernel and of the
    # inference kernel (256 accumulator registers per lane), and four per compute unit.
    mfma_loop = {}
    for name, kind in (("bf16", 0), ("int8", 1)):
        for wgs in (1, 4):
            st, rate = aser.aser_mfma_rate_probe(ctx, kind, wgs, 4000)
            ctx.check(st)
            mfma_loop["%s_%dwg_per_cu" % (name, wgs)] = round(rate, 1)
    mfma_loop["unit"] = "TFLOP/s (bf16, v_mfma_f32_32x32x16_bf16), TOP/s (int8, v_mfma_i32_32x32x32_i8)"
    # The same instructions with the operand traffic of a 256 x 256 tile around them and nothing else (32 KB of
    # LDS-direct loads per 64-byte K step and workgroup, the fragment reads, one barrier): what moving the
    # operands costs on this device, whatever the kernel does besides.
    ctx.ensure_workspace((33 << 20) + (1 << 20))
    for name, kind in (("bf16", 2), ("int8", 3)):
        st, rate = aser.aser_mfma_rate_probe(ctx, kind, 1, 4000)
        ctx.check(st)
        mfma_loop["%s_with_operand_traffic" % name] = round(rate, 1)

    _, svd_block, svd_iters = aser.aser_svd_plan(spec.m, spec.n, spec.r)
    traffic = measured_traffic()
    # fp32-class contractions of the path: algorithmic flops, and executed MFMA flops (three bf16 products per
    # fp32 product), against the bf16 dense peak and the fp32 MFMA peak
    mx = float(max(spec.m, spec.n))
    alg = {"whiten": spec.n ** 3 / 3.0,
           "reconstruct": float(spec.m) * spec.n * (spec.n + 1) + (svd_iters + 2) * 4.0 * spec.m * spec.n * svd_block
                          + (2 * svd_iters + 3) * 4.0 * mx * svd_block * svd_block}
    stage_util = {}
    for k, ms in zip(stage_names, stage_ms):
        if k in alg:
            tf = alg[k] / (ms * 1e-3) / 1e12
            stage_util[k] = {"algorithmic_flops": alg[k], "achieved_tflops": round(tf, 2),
                             "util_alg_of_bf16_peak": round(tf / BF16_PEAK_TFLOPS, 5),
                             "util_exec_of_bf16_peak": round(3.0 * tf / BF16_PEAK_TFLOPS, 5),
                             "util_alg_of_fp32_mfma_peak": round(tf / FP32_MFMA_PEAK_TFLOPS, 4)}
    out = {
        "metric": METRIC, "value": head_ms, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head_ms, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if spec.x_dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "%s: W %dx%d fp32, X %dx%d %s, W%d per-channel RTN, r=%d, f=%d" %
                               (spec.name, spec.m, spec.n, spec.tokens, spec.n, spec.x_dtype, spec.bits, spec.r, spec.f),
                   "svd_block": svd_block, "svd_iters": svd_iters, "layers_in_flight": head_n,
                   "layers_timed": head_layers,
                   "note": "value = wall clock per layer over `layers_timed` layers (`steps` rounded up to whole rounds "
                           "of `layers_in_flight`), every one a full pass from the resident "
                           "X (statistics cleared, Gram update, smoothing, RTN, whitening, reconstruction), with "
                           "`layers_in_flight` of them on the device at a time (aser_calibrate_layers); "
                           "one_layer_at_a_time_ms is the same pass with a host wait after every layer"},
        "one_layer_at_a_time_ms": ms_per_step,
        "sum_of_stage_ms": round(sum(stage_ms), 4),
        "layers_per_s": 1e3 / head_ms,
        "calibration_tokens_per_s": spec.tokens * 1e3 / head_ms,
        "stage_ms": {k: round(v, 4) for k, v in zip(stage_names, stage_ms)},
        "gram_mfma_util_pct": 100.0 * gram_tflops / BF16_PEAK_TFLOPS,
        "stage_util": stage_util,
        "layers_in_flight": in_flight,
        "whitened_error": err,
        "roofline": {"kernel": "gram_dma_kernel (Gram update G += X^T X, 256x256 lower-triangle tiles, bf16 MFMA)",
                     "bound": "mfma", "achieved": gram_tflops, "peak": BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": gram_tflops / BF16_PEAK_TFLOPS,
                     "traffic": traffic.get("gram_dma_kernel") if spec.name == "c1" else None,
                     "algorithmic_flops_per_launch": gram_flops, "avg_launch_ms": gram_ms,
                     "frac_of_mfma_only_loop": gram_tflops / mfma_loop["bf16_1wg_per_cu"],
                     "frac_of_mfma_loop_with_operand_traffic": gram_tflops / mfma_loop["bf16_with_operand_traffic"]},
        "mfma_only_loop": mfma_loop,
        "roofline_hbm": {"kernel": "rtn_kernel (per-channel RTN + target T)", "bound": "hbm", "achieved": rtn_gbs,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": rtn_gbs / HBM_PEAK_GBS,
                         "traffic": traffic.get("rtn_kernel") if spec.name == "c1" else None,
                         "algorithmic_bytes_per_launch": rtn_bytes, "avg_launch_ms": rtn_ms,
                         "plain_copy_of_as_many_bytes_gbs": round(copy_rtn_gbs, 1),
                         "frac_of_plain_copy": rtn_gbs / copy_rtn_gbs},
        "roofline_act_quant": {"kernel": "act_rtn_wave_kernel (per-token A8 quantizer of X M^-1)", "bound": "hbm",
                               "achieved": act_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": act_gbs / HBM_PEAK_GBS,
                               "traffic": None, "algorithmic_bytes_per_launch": act_bytes, "avg_launch_ms": act_ms,
                               "plain_copy_of_as_many_bytes_gbs": round(copy_act_gbs, 1),
                               "frac_of_plain_copy": act_gbs / copy_act_gbs},
    }
    if not args.no_extras:
        out["beyond_calibration"] = extras(ctx, aser, torch, spec, buf, Ws[0], X, reps)
        fwd = out["beyond_calibration"].get("compensated_forward")
        if fwd:
            fwd["roofline"]["frac_of_mfma_only_loop"] = fwd["roofline"]["achieved"] / mfma_loop["int8_1wg_per_cu"]
            fwd["roofline"]["frac_of_mfma_loop_with_operand_traffic"] = fwd["roofline"]["achieved"] / mfma_loop["int8_with_operand_traffic"]
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(spec)
    log("stage ms:", out["stage_ms"], "gram %.3f ms = %.1f TFLOP/s" % (gram_ms, gram_tflops),
        "rtn %.1f us = %.0f GB/s" % (rtn_ms * 1e3, rtn_gbs), "act quant %.1f us = %.0f GB/s" % (act_ms * 1e3, act_gbs))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
