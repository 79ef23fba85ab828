#!/usr/bin/env python3
"""Outer-step throughput of one ~100B-class pipeline stage on one MI355X.

One "step" is one full outer step of Alg. 2 (DiLoCoX) over every matrix of the stage: error
buffers and outer Nesterov update from the previous round's average, pseudo-gradients with error
compensation for K simulated workers, both compression phases (projection, quantisation,
in-memory "AllReduce" average, orthonormalisation), and the rank measurement of Alg. 3.
Inputs are synthetic (synth/), resident in HBM before the timed region.

Prints ONE JSON line (see the keys below).  `value` is stage parameters per second.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# HBM bytes per matrix element and launch from rocprofv3 FETCH_SIZE / WRITE_SIZE counter runs of
# `bench.py --probe --layers 1 --streams 1` (config 2), scaled by a 1 GiB copy in the same run
# (FETCH_SIZE reads 0.5 KiB per KiB copied, WRITE_SIZE 1.0): profiles/pmc_hbm_traffic_cfg2.txt
MEASURED_TRAFFIC_BPP = {"round_fused": 60.40, "project_q": 16.76}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_stage(cfg_id, mma, layers, device, fused, streams, plain=False, workers=0, iters=1,
                chunk=0, requant=False):
    """plain=True draws i.i.d. Gaussian replicas instead of the low-rank-plus-noise recipe (no
    library QR/GEMM kernels in the process: used for hardware-counter runs, where only the
    traffic of this library's kernels is of interest)."""
    import torch

    import synth
    from paper_2506_21263_amd.stage import MatrixState, Stage

    cfg = synth.CONFIGS[cfg_id]
    K, r = workers or cfg["K"], cfg["r"]
    mats, locals_ = [], []
    gen = torch.Generator(device="cpu")
    gen.manual_seed(1234 + cfg_id)
    t0 = time.time()
    idx = 0
    for layer in range(layers):
        for (m, n) in cfg["layer_shapes"]:
            alpha = cfg["alpha"]
            if alpha is None or alpha == "per-round":
                alpha = float(0.5 + 1.5 * torch.rand(1, generator=gen).item())
            sigma = float(synth.noise_sigma(cfg_id, m, n))
            if plain:
                th = 0.02 * torch.randn(m, n, device=device)
                dt = torch.bfloat16 if cfg["theta_l"] == "bf16" else torch.float32
                t = dict(theta_g=th, q_in=torch.randn(r, n, device=device),
                         theta_l=[(th - sigma * torch.randn(m, n, device=device)).to(dt)
                                  for _ in range(K)])
            else:
                t = synth.torch_matrix_inputs(m, n, K, r, seed=synth.seed_for(cfg_id, layer, idx),
                                              sigma=sigma, alpha=alpha, theta_l=cfg["theta_l"],
                                              device=device)
            mats.append(MatrixState(t["theta_g"], K, t["q_in"], cfg["qbits"], cfg["group"], mma))
            locals_.append(t["theta_l"])
            idx += 1
        log("generated layer %d/%d  (%.1f s, %.1f GB allocated)" %
            (layer + 1, layers, time.time() - t0, torch.cuda.memory_allocated() / 1e9))
    stage = Stage(mats, synth.LR, synth.MU, fused=fused, warm_start=True, streams=streams,
                  measure_rank=True, iters=iters, chunk=chunk, requant=requant)
    return stage, locals_


def algorithmic_bytes_per_param(kernel, K, tl_bytes, fused):
    """HBM bytes one launch of `kernel` must move per matrix element (factor traffic, a few
    per cent of it at r = 64, left out): every state read once and written once."""
    table = {
        "delta_ef": 4 + tl_bytes + 4 + 4,          # theta_g, theta_l, e in; delta out (per worker)
        "project_p": 4 * K,                         # delta of K workers, read once
        "project_q": 4 * K,
        "outer_nesterov": 20,                       # theta, v in/out; delta_hat in
        # fused: e_k in, theta_l,k in, delta_k out per worker + theta, v in/out
        "reconstruct": ((8 + tl_bytes) * K + 16) if fused else (4 + 8 * K),
        # the fused round kernel: the same, the P-phase projection rides along for free
        "round_fused": (8 + tl_bytes) * K + 16,
    }
    return table.get(kernel)


def cpu_baseline(stage, locals_, cfg_id):
    """The oracle, as it stands, on one matrix of the workload: outer steps of the smallest
    matrix shape of the stage (K workers), single thread, for about 12 s (at least two steps:
    the first applies nothing)."""
    import numpy as np
    import torch

    import synth
    from oracle import pipeline

    cfg = synth.CONFIGS[cfg_id]
    sizes = [M.m * M.n for M in stage.mats]
    a = sizes.index(min(sizes))
    M = stage.mats[a]
    theta = M.theta_g.cpu().numpy()
    q_in = M.q_in[: M.r].cpu().numpy()
    tl = []
    for x in locals_[a]:
        if x.dtype.is_floating_point and x.element_size() == 2:
            tl.append(x.view(torch.int16).cpu().numpy().view(np.uint16))
        else:
            tl.append(x.cpu().numpy())
    orc = pipeline.MatrixOracle(theta, M.K, q_in, cfg["qbits"], cfg["group"], synth.LR, synth.MU,
                                iters=stage.iters, requant=stage.requant)
    t0 = time.time()
    steps = 0
    while steps < 2 or (time.time() - t0) * (steps + 1) / steps < 12.0:
        orc.step(tl)
        orc.set_basis(orc.q_bar)
        steps += 1
    dt = (time.time() - t0) / steps
    return {"value": M.m * M.n / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": "%d outer steps of one %dx%d matrix of the stage (K=%d, r=%d, int%d/%d), "
                      "%.1f s per step" % (steps, M.m, M.n, M.K, M.r, cfg["qbits"], cfg["group"],
                                           dt)}


def quant_only(args):
    """The outer step with the quantiser as the whole compressor (the Int4-only setting of the
    paper's smaller model, Sec. 4.1): every tensor of the stage, matrices and vectors alike, is
    one flat array and one launch of dlcx_quant_round per outer step."""
    import numpy as np
    import torch

    import paper_2506_21263_amd as dlcx
    import synth
    from oracle import pipeline

    dlcx.lib()
    device = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    K = args.workers or cfg["K"]
    qbits, group = cfg["qbits"], cfg["group"]
    layers = args.layers or cfg["layers"]
    dt_l = torch.bfloat16 if cfg["theta_l"] == "bf16" else torch.float32
    hidden = min(min(s) for s in cfg["layer_shapes"])
    tensors = []
    for layer in range(layers):
        sizes = [m * n for (m, n) in cfg["layer_shapes"]]
        sizes += [4 * hidden]           # two norm weights and two biases per layer, one bucket
        for numel in sizes:
            th = 0.02 * torch.randn(numel, device=device)
            tl = [(th - 1e-3 * torch.randn(numel, device=device)).to(dt_l) for _ in range(K)]
            cb = numel // 2 if qbits == 4 else numel
            tensors.append(dict(
                numel=numel, theta=th, v=torch.zeros_like(th), tl=tl,
                ef=[torch.zeros(numel, device=device) for _ in range(K)],
                codes=[torch.empty(cb, device=device, dtype=torch.uint8) for _ in range(K)],
                scales=[torch.empty(numel // group, device=device) for _ in range(K)]))
    params = sum(t["numel"] for t in tensors)
    log("quantise-only stage: %d tensors, %.3f G params, K=%d, %.1f GB allocated" %
        (len(tensors), params / 1e9, K, torch.cuda.memory_allocated() / 1e9))
    state = {"t": 0}

    def one_step():
        state["t"] += 1
        first = state["t"] == 1
        for T in tensors:
            dlcx.dlcx_quant_round(T["numel"], qbits, group, T["tl"], T["ef"], T["theta"], T["v"],
                                  synth.LR, synth.MU, None if first else T["codes"],
                                  None if first else T["scales"], T["codes"], T["scales"],
                                  requant=args.requant)

    if args.probe:
        x = torch.empty(1 << 28, dtype=torch.float32, device=device)
        y = torch.empty_like(x)
        y.copy_(x)  # the plain copy of known size (1 GiB in, 1 GiB out) the counters are scaled by
        for _ in range(3):
            one_step()
        torch.cuda.synchronize()
        print("probe done: %d tensors, 3 steps" % len(tensors), file=sys.stderr)
        return
    for _ in range(max(args.warmup, 1)):   # the first outer step has no previous payload
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    dlcx.dlcx_profile_enable(True)
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    prof = dlcx.dlcx_profile_read()
    dlcx.dlcx_profile_enable(False)
    ms, cnt = prof["quant_round"]
    tl_bytes = 2 if cfg["theta_l"] == "bf16" else 4
    code_b = (0.5 if qbits == 4 else 1.0) + 4.0 / group
    # per worker: theta_l and delta in, delta and the new payload out, the previous payload in;
    # once: theta and v in and out
    bpp = K * (tl_bytes + 8 + 2 * code_b) + 16
    achieved = bpp * params * args.steps / (ms * 1e-3) / 1e9
    out = {
        "metric": "outer-step params/sec per stage (quantise-only compressor + avg + Nesterov)",
        "value": params / (dt / args.steps), "unit": "params/s", "n_gpus": 1,
        "steps": args.steps, "warmup": max(args.warmup, 1), "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (fp64 sums, one rounding)", "data": "synthetic",
        "config": {"workload": cfg["name"] + "-quant-only", "layers": layers,
                   "tensors": len(tensors), "params": params, "K": K, "qbits": qbits,
                   "group": group, "theta_l": cfg["theta_l"], "requant": bool(args.requant)},
        "roofline": {"kernel": "quant_round", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": None, "algorithmic_bytes_per_param_per_launch": bpp,
                     "avg_launch_ms": ms / cnt, "launches_per_step": cnt / args.steps},
        "kernels": {k: {"ms_per_step": v[0] / args.steps, "launches_per_step": v[1] / args.steps}
                    for k, v in prof.items()},
    }
    if not args.no_cpu_baseline:
        T = max(tensors, key=lambda t: t["numel"])
        th = (0.02 * np.random.default_rng(1).standard_normal(T["numel"])).astype(np.float32)
        tl = []
        for x in T["tl"]:
            tl.append(x.view(torch.int16).cpu().numpy().view(np.uint16) if x.element_size() == 2
                      else x.cpu().numpy())
        orc = pipeline.TensorOracle(th, K, qbits, group, synth.LR, synth.MU, requant=args.requant)
        t1 = time.time()
        nsteps = 0
        while nsteps < 2 or time.time() - t1 < 10.0:   # about 10 s of single-thread work
            orc.step(tl)
            nsteps += 1
        dtc = (time.time() - t1) / nsteps
        out["cpu_baseline"] = {"value": T["numel"] / dtc, "unit": "params/s", "cores": 1,
                               "kind": "oracle",
                               "sample": "%d outer steps of one tensor of %d elements (K=%d, "
                                         "int%d/%d), %.2f s per step" %
                                         (nsteps, T["numel"], K, qbits, group, dtc)}
    print(json.dumps(out), flush=True)


def mfma_peak(args):
    """Attainable bf16 matrix-core rate of this GPU (32x32x16 MFMAs, nothing competing)."""
    import torch

    import paper_2506_21263_amd as dlcx

    dlcx.lib()
    torch.cuda.set_device(0)
    wgs, iters = 256 * 8, 20000
    out = torch.empty(wgs * 256, device="cuda:0")
    rates = {}
    for name, rnd in (("small_integer_operands", False), ("random_operands", True)):
        dlcx.dlcx_mfma_peak_probe(wgs, 100, out, random_operands=rnd)
        torch.cuda.synchronize()
        dlcx.dlcx_profile_enable(True)
        for _ in range(3):
            dlcx.dlcx_mfma_peak_probe(wgs, iters, out, random_operands=rnd)
        torch.cuda.synchronize()
        ms, cnt = dlcx.dlcx_profile_read()["mfma_peak"]
        dlcx.dlcx_profile_enable(False)
        flop = wgs * 4 * iters * 8 * 32768.0
        rates[name] = {"TFLOPs": flop / (ms / cnt * 1e-3) / 1e12, "ms_per_launch": ms / cnt}
    rate = rates["random_operands"]["TFLOPs"]
    print(json.dumps({"metric": "attainable bf16 MFMA rate (v_mfma_f32_32x32x16_bf16), random operands",
                      "value": rate, "unit": "TFLOP/s", "datasheet_peak": 2500.0,
                      "frac_of_datasheet": rate / 2500.0, "rates": rates,
                      "workgroups": wgs, "mfma_per_wavefront": iters * 8}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration (synth.CONFIGS)")
    ap.add_argument("--mma", type=int, default=2, help="0 fma/fp64-acc, 1 fp32-accurate MFMA, 2 bf16 MFMA")
    ap.add_argument("--layers", type=int, default=0, help="layers resident (0 = the whole stage)")
    ap.add_argument("--unfused", action="store_true", help="separate decompress / Nesterov kernels")
    ap.add_argument("--streams", type=int, default=3, help="HIP streams the matrices are dealt to")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gemm-load", type=int, default=0,
                    help="bf16 8192^3 GEMMs issued on a second stream per outer step (config 4)")
    ap.add_argument("--graph", action="store_true",
                    help="record the steady outer step into a HIP graph and replay it (fixed ranks)")
    ap.add_argument("--workers", type=int, default=0, help="K (0 = the configuration's)")
    ap.add_argument("--quant-only", action="store_true",
                    help="quantiser as the whole compressor (no low-rank step), all tensors flat")
    ap.add_argument("--requant", action="store_true",
                    help="re-encode every average (factors, or the tensor in quantise-only mode) "
                         "to q bits before it is used")
    ap.add_argument("--chunk", type=int, default=0,
                    help="matrices per batch of a stream (0 = the stream's whole share at once)")
    ap.add_argument("--power-iters", type=int, default=1,
                    help="power iterations per round (1 = the paper's compressor)")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="measure the attainable bf16 matrix-core rate and exit")
    ap.add_argument("--probe", action="store_true",
                    help="counter run: plain random inputs, one 1 GiB copy, two steps, no timing")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE MI355X; --gpus %d is not supported "
              "(no collectives, no second GPU in this run)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.mfma_peak:
        return mfma_peak(args)
    if args.quant_only:
        return quant_only(args)

    import torch

    import paper_2506_21263_amd as dlcx
    import synth
    from paper_2506_21263_amd.stage import RankSelector

    dlcx.lib()  # fail loudly if the HIP library is missing
    device = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.config]
    layers = args.layers or cfg["layers"]
    if args.config == 4 and not args.layers:
        # K = 8 replicas of the full stage need 479 GB: time a window of 5 of the 10 identical,
        # independent layers with persistent state (value stays parameters per second)
        layers = 5
    fused = not args.unfused
    stage, locals_ = build_stage(args.config, args.mma, layers, device, fused, args.streams,
                                 plain=args.probe, workers=args.workers, iters=args.power_iters,
                                 chunk=args.chunk, requant=args.requant)
    if args.probe:
        x = torch.empty(1 << 28, dtype=torch.float32, device=device)
        y = torch.empty_like(x)
        y.copy_(x)  # the plain copy of known size (1 GiB in, 1 GiB out) the counters are scaled by
        for _ in range(2):
            stage.step(locals_)
        torch.cuda.synchronize()
        print("probe done: %d matrices, 2 steps" % len(stage.mats), file=sys.stderr)
        return
    K = args.workers or cfg["K"]
    params = stage.params()
    selector = RankSelector(stage, c=cfg.get("window", 5), r1=cfg["r"], rmin=cfg.get("rmin", 4),
                            rmax=cfg.get("rmax", cfg["r"]), H1=125)
    selector.first()
    adaptive = args.config == 3
    ranks = []
    load = None
    if args.gemm_load:
        # synthetic inner-step load: bf16 GEMMs 8192^3 on a stream of their own
        load = {"stream": torch.cuda.Stream(device=device),
                "a": torch.randn(8192, 8192, device=device, dtype=torch.bfloat16),
                "b": torch.randn(8192, 8192, device=device, dtype=torch.bfloat16),
                "c": torch.empty(8192, 8192, device=device, dtype=torch.bfloat16), "n": 0}
    log("stage: %d matrices, %.3f G params, K=%d, %.1f GB allocated" %
        (len(stage.mats), params / 1e9, K, torch.cuda.memory_allocated() / 1e9))

    use_graph = {"on": False}

    def one_step(serial=False):
        if use_graph["on"] and not serial:
            stage.replay()
            rp, r_next, _ = selector.next(stage.t + 1)
            ranks.append((rp, r_next))
            return
        if load is not None:
            with torch.cuda.stream(load["stream"]):
                for _ in range(args.gemm_load):
                    torch.matmul(load["a"], load["b"], out=load["c"])
            load["n"] += args.gemm_load
        stage.step(locals_, serial=serial)
        # Alg. 3: measure r' on this round's averages and apply the window rule; only the
        # adaptive configuration lets the result change the rank of the next compression
        rp, r_next, _ = selector.next(stage.t + 1)
        ranks.append((rp, r_next))
        if adaptive:
            for M in stage.mats:
                if r_next > M.r:  # fresh seeded columns for a basis that grows
                    M.q_bar[M.r:r_next].normal_()
                M.r = r_next
        if load is not None:
            torch.cuda.current_stream().wait_stream(load["stream"])

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    # fixed ranks and no foreign stream: the steady outer step can be recorded once into a HIP
    # graph (all launches on all streams) and replayed; measured, it changes nothing here, the
    # host is not what the step waits for
    if args.graph and not adaptive and load is None and stage.t >= 2:
        stage.capture(locals_)
        use_graph["on"] = True
        one_step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = params / (dt / args.steps)

    # per-kernel durations: the same steps again with HIP events around every launch, all on
    # one stream so that a kernel's events bracket that kernel alone
    dlcx.dlcx_profile_enable(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        one_step(serial=True)
    torch.cuda.synchronize()
    dt_prof = time.perf_counter() - t1
    prof = dlcx.dlcx_profile_read()
    dlcx.dlcx_profile_enable(False)
    tl_bytes = 2 if cfg["theta_l"] == "bf16" else 4
    kernels = {}
    for name, (ms, cnt) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
        kernels[name] = {"ms_per_step": ms / args.steps, "launches_per_step": cnt / args.steps}
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    bpp = algorithmic_bytes_per_param(dom, K, tl_bytes, fused)
    roofline = None
    if bpp is not None:
        per_worker = dom == "delta_ef"
        launches = kernels[dom]["launches_per_step"]
        # bytes of all launches of the kernel in one step / their summed duration
        total_bytes = bpp * params * (K if per_worker else 1)
        achieved = total_bytes / (kernels[dom]["ms_per_step"] * 1e-3) / 1e9
        roofline = {"kernel": dom, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "traffic": (MEASURED_TRAFFIC_BPP[dom] * params / launches
                                if dom in MEASURED_TRAFFIC_BPP and args.config == 2 else None),
                    "algorithmic_bytes_per_param_per_launch": bpp,
                    "avg_launch_ms": kernels[dom]["ms_per_step"] / launches,
                    "launches_per_step": launches}
        if dom == "round_fused" and args.mma != 0:
            # matrix-core work of the same kernel: r (reconstruction) + r K (projection)
            # multiply-adds per element, each as 3 (bf16x2) or 6 (bf16x3) bf16 piece products
            pieces = 3 if args.mma == 2 else 6
            useful = 2.0 * cfg["r"] * (1 + K) * params
            roofline["mfma"] = {
                "useful_TFLOPs": useful / (kernels[dom]["ms_per_step"] * 1e-3) / 1e12,
                "executed_bf16_TFLOPs": useful * pieces / (kernels[dom]["ms_per_step"] * 1e-3) / 1e12,
                "peak_bf16_TFLOPs": 2500.0,
                "note": "HBM-bound: %.0f executed flop per byte against a ridge of 312"
                        % (2.0 * cfg["r"] * (1 + K) * pieces / bpp)}
    # every further power iteration reads each worker's pseudo-gradient twice more
    b_alg = (14 if tl_bytes == 2 else 16) * K + 20 + 8 * K * (args.power_iters - 1)
    out = {
        "metric": "outer-step params/sec per stage (compress+avg+Nesterov)",
        "value": value, "unit": "params/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": {0: "f32 (fp64 accumulate)", 1: "bf16x3-split MFMA (fp32-accurate), f32 accumulate",
                  2: "bf16x2-split MFMA, f32 accumulate"}[args.mma],
        "data": "synthetic",
        "config": {"workload": cfg["name"], "layers": layers, "matrices": len(stage.mats),
                   "params": params, "K": K, "rank": cfg["r"], "qbits": cfg["qbits"],
                   "group": cfg["group"], "theta_l": cfg["theta_l"], "mma": args.mma,
                   "fused": fused, "streams": stage.nstreams, "hip_graph": use_graph["on"],
                   "power_iters": args.power_iters, "requant": bool(args.requant)},
        "roofline": roofline,
        "stage_hbm": {"algorithmic_bytes_per_param": b_alg,
                      "achieved_GBps": b_alg * params / (dt / args.steps) / 1e9,
                      "frac_of_8TBps": b_alg * params / (dt / args.steps) / 1e9 / HBM_PEAK_GBS},
        "kernels": kernels,
        "ms_per_step_serial_with_events": dt_prof / args.steps * 1e3,
        "rank_trace": ranks[-(2 * args.steps):][:args.steps],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(stage, locals_, args.config)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
