#!/usr/bin/env python3
"""Benchmark of the quantized DiT linear path (DAQ -> INT8 GEMM -> dequantization) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One "step" = one pass of the whole hot path over one batch of synthetic input: every
layer of the workload runs DAQ + GEMM + epilogue (fp16 in HBM -> fp16 in HBM) through
qlinear_plan_run.  Prints ONE JSON line: effective INT8 TOPS (sum of 2*M*N*K over the
layers / time), the roofline of the dominant kernel measured with events around its own
launches, and the CPU oracle timed on the host cores on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workload  # noqa: E402

INT8_PEAK_TOPS = 5033.0   # MI355X dense INT8 matrix peak (256 CUs x 2.4 GHz x 8192 op/clk)
HBM_PEAK_GBS = 8000.0
DEFAULT_WORKLOAD = "c5_stack_plan_m16384"   # the largest single-GPU configuration: 112 layers, M = 16384
POOL = 4                  # distinct activation sets rotated over the steps (different drift sigma each)
# HBM bytes per GEMM launch (reads + writes, mean over the GEMM launches of a step).  NOT measured by the run that
# prints them: they come from earlier rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of `bench.py --traffic-probe`, each
# scaled by what the same counter reads for a device-to-device copy of known size in the same run; the summary file
# under profiles/ is named beside each figure.  Keyed by (workload, forced variant, 4-bit group); absent = not measured.
TRAFFIC_BYTES_PER_LAUNCH = {
    # (2 x FETCH_SIZE + WRITE_SIZE) KiB -> bytes, mean over the launches of the workload's dominant GEMM kernel in a step
    ("c5_stack_plan_m16384", -1, 128): (176468597, "profiles/qgemm_daq_c5_stack_m16384_hbm_traffic.txt (qgemm_w4, 74 launches per step)"),
    ("c4_block_w8a8_m16384", -1, 128): (211073875, "profiles/qgemm_daq_c4_block_m16384_hbm_traffic.txt (qgemm_dma, 4 launches per step)"),
    ("c2_block_w8a8_m2048", -1, 128): (37098200, "profiles/qgemm_daq_c2_block_m2048_hbm_traffic.txt (qgemm_dma, 4 launches per step)"),
}


def mfma_probe():
    """The benchmark's own measurement aid (bench_mfma_probe.hip, its own shared object beside this file): returns
    probe(iters, blocks, sink) that enqueues the register-resident MFMA loop on torch's current stream."""
    import ctypes
    import torch
    path = os.path.join(ROOT, "libbench_mfma_probe.so")
    if not os.path.exists(path):
        from paper_2511_11446_amd import build as hip_build
        hip_build.build_bench_probe(verbose=False)
    fn = ctypes.CDLL(path).bench_mfma_probe
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]

    def probe(iters, blocks, sink):
        rc = fn(iters, blocks, sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
        if rc != 0:
            raise RuntimeError("bench_mfma_probe failed: %d" % rc)
    return probe


def build_layers(ql, torch, wl_name, w4_group=128):
    wl = workload.WORKLOADS[wl_name]
    if wl["layers"] == "bit_plan":
        descs = [(p["name"], p["K"], p["N"], p["bits"], p["block"], w4_group) for p in workload.bit_plan()]
    elif wl["layers"] == "final_plan":
        descs = [(p["name"], p["K"], p["N"], p["bits"], p["block"], p["group"] or 128) for p in workload.final_plan()]
    else:
        descs = [(n, k, o, b, 0, w4_group) for (n, k, o, b) in wl["layers"]]
    layers = []
    for name, K, N, bits, blk, group in descs:
        lw = workload.layer_weights(name, K, N, bits, wl_name, blk)
        w = ql.ql_pack_w4_host(lw["w"]) if bits == 4 else lw["w"]
        if bits == 4 and group != 128:
            lw = dict(lw, s_w=workload.w4_scales_group(N, K, group, wl_name, name, blk))
        layers.append(dict(name=name, K=K, N=N, bits=bits, group=group, w=torch.from_numpy(w).cuda(),
                           w_scale=None if lw["s_w"] is None else torch.from_numpy(lw["s_w"]).cuda(),
                           bias=torch.from_numpy(lw["bias"]).cuda(), host=lw))
    return wl, layers


def build_inputs(ql, torch, wl_name, wl, layers):
    """Per layer type one fp16 activation buffer per pool slot, drift sigma taken from the workload's schedule.
    The MLP output layer (fc2) gets the GELU of the GPU's own fc1 output of the same slot."""
    M, R = wl["M"], wl["R"]
    steps = wl["steps"]
    # every workload rotates POOL distinct input sets, so that no step finds its inputs in the caches from the step before
    sig = workload.sigma_schedule(steps) if steps > 1 else np.ones(POOL)
    slots = [int(round(i * (len(sig) - 1) / max(POOL - 1, 1))) for i in range(POOL)] if steps > 1 else list(range(POOL))
    types = {}
    for l in layers:
        types.setdefault(l["name"], (l["K"], l["N"]))
    pool = []
    for s in slots:
        x = {}
        for name, (K, N) in types.items():
            if name == "fc2" and "fc1" in types:
                continue
            x[name] = torch.from_numpy(workload.activations(M, K, wl_name, name, s, sigma=float(sig[s]))).cuda()
        if "fc2" in types and "fc1" in types:
            fc1 = next(l for l in layers if l["name"] == "fc1")
            if fc1["bits"] == 16:
                y1 = ql.qlinear_f16(x["fc1"], fc1["w"], fc1["bias"])
            elif fc1["bits"] == 8:
                y1 = ql.qlinear_w8a8(x["fc1"], R, fc1["w"], fc1["w_scale"], fc1["bias"])
            else:
                y1 = ql.qlinear_w4a8(x["fc1"], R, fc1["w"], fc1["w_scale"], fc1["bias"], group=fc1["group"])
            x["fc2"] = torch.nn.functional.gelu(y1.float(), approximate="tanh").half()   # input preparation only
            del y1
        elif "fc2" in types:
            K = types["fc2"][0]
            x["fc2"] = torch.from_numpy(workload.gelu_tanh_f16(
                workload.activations(M, K, wl_name, "fc2", s, sigma=float(sig[s])))).cuda()
        pool.append(x)
    return pool, [float(sig[s]) for s in slots]


def cpu_baseline(wl_name, wl, layers, budget_rows=8192, min_seconds=10.0, max_passes=32):
    """The oracle as it stands, row-parallel over the host cores, on the first rows of the workload (one launch of every
    distinct layer kind); whole passes over that sample are repeated until about ten seconds of CPU work have been timed
    (a pass over 8192 rows of the eight layer kinds of the 112-layer stack takes about 13 s on 16 threads)."""
    import oracle
    oracle.build()
    M, R = wl["M"], wl["R"]
    uniq = {}
    for l in layers:
        uniq.setdefault((l["name"], l["bits"]), l)
    rows = min(M, budget_rows)
    Rs = R if (R <= rows and rows % R == 0) else rows   # a scale block larger than the sample becomes the sample
    threads = oracle.max_threads()
    prepared = []
    for l in uniq.values():
        x = workload.activations(rows, l["K"], wl_name, l["name"], "cpu")
        lw = l["host"]
        w = oracle.pack_w4(lw["w"]) if l["bits"] == 4 else lw["w"]
        prepared.append((l, x, w, lw))
    t_total, macs, passes = 0.0, 0, 0
    while passes < max_passes and (passes == 0 or t_total < min_seconds):
        for l, x, w, lw in prepared:
            t0 = time.perf_counter()
            if l["bits"] == 16:
                oracle.linear_f16(x, w, lw["bias"], nthreads=threads)
            elif l["bits"] == 8:
                oracle.qlinear_w8a8(x, Rs, w, lw["s_w"], lw["bias"], nthreads=threads, want_debug=False)
            else:
                if l["group"] == 128:
                    oracle.qlinear_w4a8(x, Rs, w, lw["s_w"], lw["bias"], nthreads=threads, want_debug=False)
                else:
                    qc, sc = oracle.daq(x, Rs, nthreads=threads)
                    oracle.epilogue_w4(oracle.gemm_w4g(qc, w, l["group"], nthreads=threads), sc, Rs, l["w_scale"].cpu().numpy(),
                                       lw["bias"])
            t_total += time.perf_counter() - t0
            macs += rows * l["K"] * l["N"]
        passes += 1
    return {"value": 2.0 * macs / t_total / 1e12, "unit": "TOPS", "cores": threads, "kind": "oracle",
            "sample": "first %d of %d rows through %d distinct layers (%s), %d pass(es), %.1f s" %
                      (rows, M, len(uniq), ",".join("%s/w%d" % k for k in uniq), passes, t_total),
            "seconds": t_total}


def planner_demo(ql, torch, args):
    """Per-layer latencies measured on this GPU -> ql_plan_greedy (Algorithm 2, Phase A) -> the chosen plan timed through the
    plan runner.  Sensitivities and drifts are seeded stand-ins (the paper measures them on its trained model): drift large
    at the first steps and decaying, sensitivity highest in the first and last blocks."""
    M, R, T = 16384, 1, 50
    stream = torch.cuda.current_stream()

    def timed(fn, reps=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record(stream)
        for _ in range(reps):
            fn()
        a1.record(stream)
        torch.cuda.synchronize()
        return a0.elapsed_time(a1) / reps * 1e3      # us

    lat, dev = {}, {}
    for name, K, N in workload.BLOCK_LAYERS:
        x = torch.from_numpy(workload.activations(M, K, "planner", name)).cuda()
        y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        ws = ql.workspace(ql.qlinear_workspace_bytes(M, K, R))
        for bits in (16, 8, 4):
            lw = workload.layer_weights(name, K, N, bits, "planner")
            w = torch.from_numpy(ql.ql_pack_w4_host(lw["w"]) if bits == 4 else lw["w"]).cuda()
            sw = None if bits == 16 else torch.from_numpy(lw["s_w"]).cuda()
            b = torch.from_numpy(lw["bias"]).cuda()
            dev[(name, bits)] = (w, sw, b)
            if bits == 16:
                lat[(name, bits)] = timed(lambda: ql.qlinear_f16(x, w, b, y=y))
            elif bits == 8:
                lat[(name, bits)] = timed(lambda: ql.qlinear_w8a8(x, R, w, sw, b, y=y, ws=ws))
            else:
                lat[(name, bits)] = timed(lambda: ql.qlinear_w4a8(x, R, w, sw, b, y=y, ws=ws))
    g = workload.rng("planner-demo")
    drift = 4.0 * np.exp(-np.arange(T) / 6.0) + 0.05 + 0.02 * g.random(T)
    descs, layers = [], []
    for blk in range(workload.N_BLOCKS):
        for name, K, N in workload.BLOCK_LAYERS:
            sens = 0.2 + 1.5 * max(0.0, 1.0 - min(blk, workload.N_BLOCKS - 1 - blk) / 4.0) + 0.3 * g.random()
            floor = lat[(name, 4)]
            layers.append(dict(bits=[16, 8, 4], c_lat=[T * (lat[(name, b)] - floor) for b in (16, 8, 4)],
                               c_mem=[N * K * b / 8.0 for b in (16, 8, 4)], sensitivity=sens))
            descs.append((name, K, N))
    c_step = np.full(T, sum(lat[(n, 4)] for n, _, _ in descs))
    full_lat = float(c_step.sum() + sum(l["c_lat"][0] for l in layers))
    full_mem = float(sum(l["c_mem"][0] for l in layers))
    B_lat, B_mem = 0.45 * full_lat, 0.40 * full_mem
    plan = ql.plan_greedy(drift, c_step, layers, B_lat, B_mem, 200000, eps=1e-9)
    kept = np.flatnonzero(plan["kept"])
    # run one step of the chosen plan
    pl, xs, ys = [], [], []
    xbuf = {n: torch.from_numpy(workload.activations(M, K, "planner", n)).cuda() for n, K, N in workload.BLOCK_LAYERS}
    ybuf = {n: torch.empty((M, N), dtype=torch.float16, device="cuda") for n, K, N in workload.BLOCK_LAYERS}
    for (name, K, N), bits in zip(descs, plan["bits"].tolist()):
        w, sw, b = dev[(name, bits)]
        pl.append(dict(K=K, N=N, bits=bits, group=128, w=w, w_scale=sw, bias=b))
        xs.append(xbuf[name])
        ys.append(ybuf[name])
    P = ql.Plan(pl, M_max=M)
    ws = ql.workspace(P.workspace_bytes(M, R))
    step_us = timed(lambda: P.run(xs, ys, M, R, ws), reps=5)
    counts = {b: int((plan["bits"] == b).sum()) for b in (16, 8, 4)}
    print(json.dumps({"planner": "Algorithm 2 Phase A on latencies measured by this library", "M": M, "T": T,
                      "measured_layer_us": {"%s/w%d" % k: v for k, v in lat.items()},
                      "budget": {"latency_us": B_lat, "memory_bytes": B_mem, "of_full": [0.45, 0.40]},
                      "plan_width_counts": counts, "kept_steps": int(len(kept)), "first_kept": kept[:8].tolist(),
                      "feasible": plan["feasible"], "C_lat_us": plan["C_lat"], "C_mem_bytes": plan["C_mem"],
                      "predicted_step_us": float(sum(lat[(n, b)] for (n, _, _), b in zip(descs, plan["bits"].tolist()))),
                      "measured_step_us": step_us}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(workload.WORKLOADS))
    ap.add_argument("--variant", type=int, default=-1, help="force a GEMM tile variant (sweeps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true")
    ap.add_argument("--daq-p-ppm", type=int, default=None,
                    help="percentile-clipped DAQ (eq. (4) as printed): p in parts per million, e.g. 999000; default: absmax")
    ap.add_argument("--a-bits", type=int, default=8, help="activation code width for --daq-p-ppm (Step 6 time-bin policy)")
    ap.add_argument("--w4-group", type=int, default=128,
                    help="k per weight scale of the 4-bit layers (the plan's other group sizes: 64, 192, 288 ...)")
    ap.add_argument("--fused-block", action="store_true",
                    help="time one block with GELU (fc1) and gated residuals (proj, fc2) folded into the epilogues, "
                         "against the same layers followed by separate elementwise kernels")
    ap.add_argument("--planner", action="store_true",
                    help="Algorithm 2 Phase A on MEASURED costs: time every layer type at 16/8/4-bit weights with this library, "
                         "let ql_plan_greedy choose widths and kept timesteps under a latency and a memory budget, then time "
                         "one step of the chosen plan through qlinear_plan_run")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: a few steps of the workload plus a device copy of known size, no timing")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (every GPU box here has one); --gpus %d is not supported. "
              "The path shards by rows (whole samples) with no exchange between GPUs." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_11446_amd as ql
    ql.ensure_built()   # compiles only if no built library is there
    ql.lib()            # raises if the HIP library is missing: there is no fallback
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    ql.set_gemm_variant(args.variant)

    if args.planner:
        planner_demo(ql, torch, args)
        return

    wl, layers = build_layers(ql, torch, args.workload, args.w4_group)
    M, R = wl["M"], wl["R"]
    big = M >= 8192
    steps = args.steps if args.steps is not None else (wl["steps"] if wl["steps"] > 1 else (100 if not big else 20))
    warmup = args.warmup
    pool, sigmas = build_inputs(ql, torch, args.workload, wl, layers)
    plan = ql.Plan([dict(K=l["K"], N=l["N"], bits=l["bits"], group=l["group"], w=l["w"], w_scale=l["w_scale"], bias=l["bias"])
                    for l in layers], M_max=M)
    ws = ql.workspace(plan.workspace_bytes(M, R))
    y_by_type = {}
    for l in layers:
        if l["name"] not in y_by_type:
            y_by_type[l["name"]] = torch.empty((M, l["N"]), dtype=torch.float16, device="cuda")
    import ctypes
    L = len(layers)
    xs_pool = [(ctypes.c_void_p * L)(*[slot[l["name"]].data_ptr() for l in layers]) for slot in pool]
    ys = (ctypes.c_void_p * L)(*[y_by_type[l["name"]].data_ptr() for l in layers])
    stream = torch.cuda.current_stream()
    sptr = ctypes.c_void_p(stream.cuda_stream)
    ops_per_step = sum(2.0 * M * l["N"] * l["K"] for l in layers)

    if args.traffic_probe:
        # counters are read per dispatch: 3 steps of the workload, then 3 copies of 256 MiB (read 256 MiB, write 256 MiB)
        for i in range(3):
            plan.run_ptrs(xs_pool[i % len(pool)], ys, M, R, ws, sptr)
        torch.cuda.synchronize()
        src = torch.ones(128 * 1024 * 1024, dtype=torch.float16, device="cuda")
        dst = torch.empty_like(src)
        for i in range(3):
            torch.mul(src, 1.0, out=dst)   # an elementwise kernel: 256 MiB read, 256 MiB written
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": args.workload, "copy_bytes_read": src.numel() * 2,
                          "copy_bytes_written": src.numel() * 2, "steps": 3}))
        return

    if args.fused_block:
        # Block glue (Section 6 counts residual additions in the latency): one DiT block's four linears with
        # proj/fc2 -> gated residual, fc1 -> GELU.  Both sequences are captured into a HIP graph and replayed.
        tokens = 256 if M % 256 == 0 else M
        by = {l["name"]: l for l in layers}
        names = [n for n in ("qkv", "proj", "fc1", "fc2") if n in by]
        x0 = pool[0]
        hid = by["proj"]["N"]
        resid = torch.randn((M, hid), device="cuda", dtype=torch.float16)
        gate = torch.randn((M // tokens, hid), device="cuda", dtype=torch.float16)
        outs = {n: torch.empty((M, by[n]["N"]), dtype=torch.float16, device="cuda") for n in names}
        wsl = ql.workspace(plan.workspace_bytes(M, R))

        def layer(n, **kw):
            l = by[n]
            return ql.qlinear_fused(x0[n], R, l["w"], l["w_scale"], l["bias"], bits=l["bits"], group=l["group"],
                                    y=outs[n], ws=wsl, **kw)

        def fused():
            layer("qkv")
            layer("proj", residual=resid, gate=gate, gate_rows=tokens)
            layer("fc1", act=ql.ACT_GELU_TANH)
            layer("fc2", residual=resid, gate=gate, gate_rows=tokens)

        tmp = torch.empty((M, hid), dtype=torch.float16, device="cuda")
        g3 = gate.repeat_interleave(tokens, dim=0)

        def unfused():
            layer("qkv")
            layer("proj")
            torch.addcmul(resid, g3, outs["proj"], out=tmp)
            layer("fc1")
            torch.nn.functional.gelu(outs["fc1"], approximate="tanh")
            layer("fc2")
            torch.addcmul(resid, g3, outs["fc2"], out=tmp)

        def timed(fn, reps=10):
            fn()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(reps):
                    fn()
            g.replay()
            torch.cuda.synchronize()
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record(stream)
            g.replay()
            a1.record(stream)
            torch.cuda.synchronize()
            return a0.elapsed_time(a1) / reps * 1e3

        tf, tu = timed(fused), timed(unfused)
        # LayerNorm + modulation in the DAQ prologue (what feeds qkv and fc1) against LayerNorm, modulation and DAQ as
        # separate kernels (PyTorch's layer_norm and addcmul, then daq_quantize)
        xr = torch.randn((M, hid), device="cuda", dtype=torch.float16)
        shift = torch.randn((M // tokens, hid), device="cuda", dtype=torch.float16)
        scale = torch.randn((M // tokens, hid), device="cuda", dtype=torch.float16) * 0.3
        sh3, sc3 = shift.repeat_interleave(tokens, dim=0), (1.0 + scale).repeat_interleave(tokens, dim=0)
        qb = torch.empty((M, hid), dtype=torch.int8, device="cuda")
        sb = torch.empty((M,), dtype=torch.float32, device="cuda")
        lib, vp = ql.lib(), ctypes.c_void_p
        lib.daq_quantize_ln.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, vp, vp, ctypes.c_int64, ctypes.c_float,
                                        vp, vp, vp, vp, ctypes.c_size_t, vp]

        def ln_fused():
            rc = lib.daq_quantize_ln(vp(xr.data_ptr()), M, hid, 1, vp(shift.data_ptr()), vp(scale.data_ptr()), tokens, 1e-6, None,
                                     vp(qb.data_ptr()), vp(sb.data_ptr()), None, 0, vp(torch.cuda.current_stream().cuda_stream))
            if rc != 0:
                raise RuntimeError("daq_quantize_ln failed: %d" % rc)

        def ln_separate():
            h = torch.nn.functional.layer_norm(xr, (hid,), eps=1e-6)
            h = torch.addcmul(sh3, h, sc3)
            ql.daq_quantize(h, 1, qb, sb)

        t_lnf, t_lns = timed(ln_fused), timed(ln_separate)
        # fc1's epilogue leaves the row maxima of its output; fc2's DAQ starts from them (one scale per token, and one
        # per image of `tokens` rows, where the separate DAQ needs a pass of its own to find the maximum)
        rowmax = torch.zeros((M,), dtype=torch.int32, device="cuda")
        f1, kf2 = outs["fc1"], by["fc2"]["K"]
        qf = torch.empty((M, kf2), dtype=torch.int8, device="cuda")
        sf = torch.empty((M,), dtype=torch.float32, device="cuda")
        dws = ql.workspace(ql.daq_workspace_bytes(M, kf2, tokens))
        t_fc1 = timed(lambda: layer("fc1", act=ql.ACT_GELU_TANH))
        t_fc1_rm = timed(lambda: layer("fc1", act=ql.ACT_GELU_TANH, row_absmax=rowmax))
        side = {"fc1_gelu_us": t_fc1, "fc1_gelu_with_row_absmax_us": t_fc1_rm}
        for rr in (1, tokens):
            side["fc2_daq_R%d_us" % rr] = timed(lambda: ql.daq_quantize(f1, rr, qf, sf, dws))
            side["fc2_daq_from_row_absmax_R%d_us" % rr] = timed(lambda: ql.daq_quantize_rowmax(f1, rr, rowmax, qf, sf, dws))
        print(json.dumps({"metric": "one block's four linears with GELU and gated residuals", "unit": "us",
                          "fused_epilogues_us": tf, "separate_elementwise_kernels_us": tu, "speedup": tu / tf,
                          "layernorm_modulate_daq_one_kernel_us": t_lnf, "layernorm_modulate_then_daq_us": t_lns,
                          "row_absmax_side_output": side,
                          "config": {"workload": args.workload, "M": M, "rows_per_scale": R, "tokens_per_gate_row": tokens}}))
        return

    robust = args.daq_p_ppm is not None

    def run_step(i):
        if robust:
            plan.run_ptrs_robust(xs_pool[i % len(pool)], ys, M, R, args.daq_p_ppm, args.a_bits, ws, sptr)
        else:
            plan.run_ptrs(xs_pool[i % len(pool)], ys, M, R, ws, sptr)

    def run_daq(x, q, sa, dws):
        if robust:
            ql.daq_quantize_robust(x, R, args.daq_p_ppm, args.a_bits, q, sa, dws)
        else:
            ql.daq_quantize(x, R, q, sa, dws)

    # The clocks take tens of milliseconds of load to settle (the first 50 steps of the M = 16384 block run 8 % slower
    # than the rest): before the W warm-up steps, run the step for at least 0.15 s of wall time (untimed preparation).
    settle, t_w0 = 0, time.perf_counter()
    while time.perf_counter() - t_w0 < 0.15:
        for _ in range(5):
            run_step(settle)
            settle += 1
        torch.cuda.synchronize()
    if warmup is None:
        warmup = 10 if not big else 3
    for i in range(warmup):
        run_step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall0 = time.perf_counter()
    e0.record(stream)
    for i in range(steps):
        run_step(i)
    e1.record(stream)
    torch.cuda.synchronize()
    t_wall = time.perf_counter() - t_wall0
    ms = e0.elapsed_time(e1)
    ms_per_step = ms / steps
    tops = ops_per_step / (ms_per_step * 1e-3) / 1e12
    # median over individually timed steps (the paper's protocol quotes averages of synchronized events; the
    # event pairs add a little per step, so the headline value stays the average over the uninterrupted run)
    n_med = min(steps, 100)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_med + 1)]
    evs[0].record(stream)
    for i in range(n_med):
        run_step(i)
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    ms_median = float(np.median([evs[i].elapsed_time(evs[i + 1]) for i in range(n_med)]))

    # ---- per-kernel breakdown: for every distinct layer, `reps` launches of the DAQ kernel and `reps` launches of the
    # GEMM kernel, each batch captured into a HIP graph (back-to-back on the stream, no host time between them) and
    # timed with events around the replay on that same stream
    roofline = None
    breakdown = {}
    mfma_ceiling = None
    if not args.no_breakdown:
        reps = 20 if not big else 10

        graph_ok = [True]

        def timed_graph(fn):
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            if graph_ok[0]:
                try:
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        for _ in range(reps):
                            fn()
                    g.replay()
                    torch.cuda.synchronize()
                    a0.record(stream)
                    g.replay()
                    a1.record(stream)
                    torch.cuda.synchronize()
                    return a0.elapsed_time(a1) * 1e-3 / reps
                except Exception as e:   # no graph capture on this stack: plain back-to-back launches instead
                    print("bench.py: HIP graph capture unavailable (%s); timing plain launch loops" % e, file=sys.stderr)
                    graph_ok[0] = False
                    torch.cuda.synchronize()
            fn()
            torch.cuda.synchronize()
            a0.record(stream)
            for _ in range(reps):
                fn()
            a1.record(stream)
            torch.cuda.synchronize()
            return a0.elapsed_time(a1) * 1e-3 / reps

        def kind(l):
            return (l["name"], l["bits"]) if l["bits"] != 4 or l["group"] == args.w4_group else (l["name"], "4g%d" % l["group"])

        uniq = {}
        for l in layers:
            uniq.setdefault(kind(l), l)
        counts = {}
        for l in layers:
            counts[kind(l)] = counts.get(kind(l), 0) + 1
        gemm_time, gemm_ops, gemm_n, daq_time, daq_bytes, daq_n = 0.0, 0.0, 0, 0.0, 0.0, 0
        fam = {}   # GEMM kernel family -> [time per step, ops per step, launches per step]
        fam_name = {8: "qgemm_dma, 8-bit weights", 4: "qgemm_w4 / qgemm_mfma, 4-bit weights", 16: "qgemm_dma, FP16 operands"}
        for key, l in uniq.items():
            x = pool[0][l["name"]]
            q = torch.empty((M, l["K"]), dtype=torch.int8, device="cuda")
            sa = torch.empty((M // R,), dtype=torch.float32, device="cuda")
            dws = ql.workspace(ql.daq_workspace_bytes(M, l["K"], R))
            y = torch.empty((M, l["N"]), dtype=torch.float16, device="cuda")
            if l["bits"] == 16:
                # a layer left in FP16: no DAQ; the "GEMM" is the whole layer on the fp16 input
                gfn = (lambda q_, sa_, R_, w_, ws_, b_, y=None, _x=x: ql.qlinear_f16(_x, w_, b_, y=y))
            elif l["bits"] == 8:
                gfn = ql.qgemm_w8a8
            else:
                gfn = (lambda *a, _g=l["group"], **kw: ql.qgemm_w4a8(*a, group=_g, **kw))
            # eager once (also the comparison for the graph replays below)
            run_daq(x, q, sa, dws)
            gfn(q, sa, R, l["w"], l["w_scale"], l["bias"], y=y)
            torch.cuda.synchronize()
            q_ref, y_ref = q.clone(), y.clone()
            td = timed_graph(lambda: run_daq(x, q, sa, dws)) if l["bits"] != 16 else 0.0
            tg = timed_graph(lambda: gfn(q, sa, R, l["w"], l["w_scale"], l["bias"], y=y))
            if not (torch.equal(q, q_ref) and torch.equal(y, y_ref)):
                raise RuntimeError("graph replay of %s/w%s differs from the eager launch" % key)
            ops = 2.0 * M * l["N"] * l["K"]
            dbytes = 3.0 * M * l["K"] + 4.0 * (M // R)
            breakdown["%s/w%s" % key] = {"daq_us": td * 1e6, "gemm_us": tg * 1e6, "gemm_tops": ops / tg / 1e12,
                                          "daq_gbs": (dbytes / td / 1e9) if td else None, "launches_per_step": counts[key]}
            gemm_time += tg * counts[key]
            gemm_ops += ops * counts[key]
            gemm_n += counts[key]
            f = fam.setdefault(l["bits"], [0.0, 0.0, 0])
            f[0] += tg * counts[key]
            f[1] += ops * counts[key]
            f[2] += counts[key]
            daq_time += td * counts[key]
            daq_bytes += (dbytes if td else 0.0) * counts[key]
            daq_n += counts[key] if td else 0
            del q, sa, y, q_ref, y_ref
        # the matrix cores' own ceiling on this machine: a register-resident MFMA loop, 2 workgroups per CU
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        cus = torch.cuda.get_device_properties(0).multi_processor_count
        probe = mfma_probe()
        pops = 2.0 * 32 * 32 * 32 * 4 * 4096 * 4 * (2 * cus)
        for _ in range(2):
            probe(4096, 2 * cus, sink)
        torch.cuda.synchronize()
        a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a0.record(stream)
        for _ in range(5):
            probe(4096, 2 * cus, sink)
        a1.record(stream)
        torch.cuda.synchronize()
        mfma_ceiling = 5 * pops / (a0.elapsed_time(a1) * 1e-3) / 1e12
        traffic = TRAFFIC_BYTES_PER_LAUNCH.get((args.workload, args.variant, args.w4_group))
        # the dominant kernel = the GEMM family with the largest share of a step (the DAQ kernel if it outweighs them all)
        dom = max(fam, key=lambda b: fam[b][0])
        if fam[dom][0] >= daq_time:
            t_dom, ops_dom, n_dom = fam[dom]
            peak = INT8_PEAK_TOPS if dom != 16 else 2500.0
            ach = ops_dom / t_dom / 1e12
            roofline = {"bound": "mfma", "kernel": fam_name[dom] + " (GEMM + dequantization): its launches of a step",
                        "achieved": ach, "peak": peak, "unit": "TOP/s" if dom != 16 else "TFLOP/s", "frac": ach / peak,
                        "avg_launch_us": t_dom / n_dom * 1e6, "ops_per_launch": ops_dom / n_dom,
                        "launches_per_step": n_dom, "share_of_gemm_time": t_dom / gemm_time,
                        "traffic": traffic[0] if traffic else None,
                        "traffic_source": traffic[1] if traffic else None}
        else:
            ach = daq_bytes / daq_time / 1e9
            roofline = {"bound": "hbm", "kernel": "daq_rows_cached (DAQ pass), all layers of a step", "achieved": ach,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                        "avg_launch_us": daq_time / daq_n * 1e6, "bytes_per_launch": daq_bytes / daq_n,
                        "traffic": None}
        roofline["by_kernel"] = {fam_name[b]: {"tops": v[1] / v[0] / 1e12, "frac_of_peak": v[1] / v[0] / 1e12 / (INT8_PEAK_TOPS if b != 16 else 2500.0),
                                               "us_per_step": v[0] * 1e6, "launches_per_step": v[2]} for b, v in fam.items()}
        roofline["daq_hbm_gbs"] = (daq_bytes / daq_time / 1e9) if daq_time else None
        roofline["daq_us_per_step"] = daq_time * 1e6
        roofline["gemm_only_tops"] = gemm_ops / gemm_time / 1e12
        roofline["gemm_only_frac"] = gemm_ops / gemm_time / 1e12 / INT8_PEAK_TOPS
        roofline["measured_mfma_only_tops"] = mfma_ceiling
        roofline["frac_of_measured_mfma"] = gemm_ops / gemm_time / 1e12 / mfma_ceiling

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(args.workload, wl, layers)

    out = {
        "metric": "effective INT8 TOPS for DAQ+qlinear on DiT-XL/2 shapes (sum 2MNK / time, fp16 in -> fp16 out)",
        "value": tops, "unit": "TOPS", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "pct_int8_mfma_peak": 100.0 * tops / INT8_PEAK_TOPS,
        "pct_measured_mfma_only": (100.0 * tops / mfma_ceiling) if mfma_ceiling else None,
        "config": {"workload": args.workload, "M": M, "rows_per_scale": R, "layers": L,
                   "w4_layers": sum(l["bits"] == 4 for l in layers), "activation_sets_rotated": len(pool),
                   "sigmas": sigmas, "gemm_variant": args.variant,
                   "w4_group": args.w4_group,
                   "daq": ("percentile p_ppm=%d a_bits=%d" % (args.daq_p_ppm, args.a_bits)) if robust else "absmax a_bits=8"},
        "ms_per_step_median": ms_median,
        "clock_settle_steps": settle,
        "inputs": "%d input sets rotated over the steps" % len(pool),
        "host_wall_ms_per_step": t_wall / steps * 1e3,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "breakdown": breakdown,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
