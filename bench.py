#!/usr/bin/env python3
"""Outer-step throughput of one ~100B-class pipeline stage on one MI355X.

One "step" is one full outer step of Alg. 2 (DiLoCoX) over every matrix of the stage: error
buffers and outer Nesterov update from the previous round's average, pseudo-gradients with error
compensation for K simulated workers, both compression phases (projection, quantisation,
in-memory "AllReduce" average, orthonormalisation), and the rank measurement of Alg. 3.
Inputs are synthetic (synth/), resident in HBM before the timed region.

Prints ONE JSON line (see the keys below).  `value` is stage parameters per second.  The default
run (config 2) appends `other_configs`: the OPT-1.3B-shaped stage, its quantise-only form and the
512 x 512 case replayed as a HIP graph, each built, timed for a few steps and freed in turn.
"""
import argparse
import copy
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
# HBM bytes per matrix element and launch of the two sweeping kernels from rocprofv3 counter runs
# of `bench.py --probe --layers 1 --streams 1` (config 2).  Round kernel: TCC_EA0_RDREQ (128-byte
# requests) and TCC_EA0_WRREQ_64B over the stage's mix of shapes,
# profiles/pmc_memory_system_round_kernel_vs_flat_sweep_cfg2.txt; Q kernel: FETCH_SIZE / WRITE_SIZE
# scaled by a 1 GiB copy in the same run, profiles/pmc_hbm_traffic_cfg2.txt.  The counters cannot
# be read from inside a timed run, so the figures of those profiles are quoted.
MEASURED_TRAFFIC_BPP = {"round_fused": 59.17, "project_q": 16.76}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_stage(cfg_id, mma, layers, device, fused, streams, plain=False, workers=0, iters=1,
                chunk=0, requant=False, keep_uv=False, stream_pool=None):
    """plain=True draws i.i.d. Gaussian replicas instead of the low-rank-plus-noise recipe (no
    library QR/GEMM kernels in the process: used for hardware-counter runs, where only the
    traffic of this library's kernels is of interest).  keep_uv keeps what a later round's
    replicas are drawn from (adaptive configuration)."""
    import torch

    import synth
    from paper_2506_21263_amd.stage import MatrixState, Stage

    cfg = synth.CONFIGS[cfg_id]
    K, r = workers or cfg["K"], cfg["r"]
    mats, inputs = [], []
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
                                              device=device, keep_uv=keep_uv)
            mats.append(MatrixState(t["theta_g"], K, t["q_in"], cfg["qbits"], cfg["group"], mma))
            inputs.append(t)
            idx += 1
        log("generated layer %d/%d  (%.1f s, %.1f GB allocated)" %
            (layer + 1, layers, time.time() - t0, torch.cuda.memory_allocated() / 1e9))
    stage = Stage(mats, synth.LR, synth.MU, fused=fused, warm_start=True, streams=streams,
                  measure_rank=True, iters=iters, chunk=chunk, requant=requant,
                  stream_pool=stream_pool)
    return stage, inputs, gen


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


# ---------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, on the machine's host cores
# ---------------------------------------------------------------------------------------------
def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg_id, K, r, iters=1, requant=False, target_elems=1 << 21):
    """The oracle (plain C, one thread per matrix, nothing tuned) on a bounded sample of the
    stage: for every distinct matrix shape one slab of whole rows -- m_s x n with the shape's own
    n, the configuration's K, rank, quantiser and replica type, about 2 M elements -- stepped
    three times (the first step has no feedback and no update and is left out of the timing).
    1 thread: the slabs one after the other.  All cores: independent slabs side by side, one
    thread each (the arithmetic per matrix is unchanged, so are its results).  The stage figure
    extrapolates the per-element rate of each shape over the stage's matrices of that shape,
    which are independent."""
    import threading

    import numpy as np

    import synth
    from oracle import pipeline

    cfg = synth.CONFIGS[cfg_id]
    shapes = []
    for s in synth.stage_shapes(cfg_id):
        if s not in shapes:
            shapes.append(s)
    counts = {s: synth.stage_shapes(cfg_id).count(s) for s in shapes}
    group = cfg["group"]

    def slab_rows(m, n):
        rows = max(target_elems // n, r, group)
        rows = (rows + group - 1) // group * group
        return min(rows, m)

    def make(shape, seed):
        m, n = shape
        ms = slab_rows(m, n)
        alpha = cfg["alpha"] if isinstance(cfg["alpha"], float) else 1.0
        inp = synth.MatrixInputs(ms, n, K, min(r, ms, n), seed=seed,
                                 sigma=float(synth.noise_sigma(cfg_id, m, n)), alpha=alpha,
                                 theta_l=cfg["theta_l"])
        orc = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, cfg["qbits"], group, synth.LR,
                                    synth.MU, iters=iters, requant=requant)
        return inp, orc, ms * n

    def make_raw(inp, steps):
        # the replicas' raw pseudo-gradients of every round, drawn before anything is timed
        return [[inp.raw_pseudo_gradient(t, i) for i in range(K)] for t in range(1, steps + 1)]

    def run(inp, orc, raw, barrier=None):
        times = []
        for t in range(1, len(raw) + 1):
            tl = []
            for i in range(K):   # theta_l,i = cast(theta_g - G_i), as synth.MatrixInputs does
                x = (orc.theta.astype(np.float64) - raw[t - 1][i]).astype(np.float32)
                tl.append(synth.f32_to_bf16_bits(x) if cfg["theta_l"] == "bf16" else x)
            if barrier is not None and t == 2:
                barrier.wait()
            t0 = time.perf_counter()
            orc.step(tl)
            orc.set_basis(orc.q_bar)
            times.append(time.perf_counter() - t0)
        return times

    # ---- one thread
    per_shape, serial_batch = [], 0.0
    for a, shape in enumerate(shapes):
        inp, orc, elems = make(shape, 7000 + a)
        times = run(inp, orc, make_raw(inp, 3))
        dt = sum(times[1:]) / 2.0
        serial_batch += sum(times[1:])
        per_shape.append({"shape": "%dx%d" % shape, "slab": "%dx%d" % (inp.m, inp.n),
                          "s_per_step": dt, "params_per_s": elems / dt})
    stage_params = sum(m * n * c for (m, n), c in counts.items())
    stage_s_1t = sum(counts[s] * s[0] * s[1] / p["params_per_s"] for s, p in zip(shapes, per_shape))
    value_1t = stage_params / stage_s_1t
    # ---- all host cores: independent slabs side by side, one thread each
    cores_total = os.cpu_count() or 1
    try:
        cores_total = min(cores_total, len(os.sched_getaffinity(0)))
    except AttributeError:
        pass
    env_cap = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)  # the machine's CPU share, if stated
    threads = max(1, min(cores_total, env_cap) if env_cap > 0 else cores_total)
    tasks = [make(shapes[i % len(shapes)], 7100 + i) for i in range(threads)]
    raws = [make_raw(task[0], 3) for task in tasks]
    barrier = threading.Barrier(threads + 1, timeout=900)
    done = []

    def worker(task, raw):
        run(task[0], task[1], raw, barrier)
        done.append(time.perf_counter())

    ths = [threading.Thread(target=worker, args=(task, raw)) for task, raw in zip(tasks, raws)]
    for th in ths:
        th.start()
    barrier.wait()
    t0 = time.perf_counter()
    for th in ths:
        th.join()
    wall = max(done) - t0
    # the same batch of slabs, one after the other, would take threads / len(shapes) times the
    # serial batch measured above
    speedup = (threads / float(len(shapes))) * serial_batch / wall
    value_all = value_1t * speedup
    return {"value": value_all, "unit": "params/s", "cores": threads, "kind": "oracle",
            "value_1t": value_1t, "value_all": value_all, "cores_total": cores_total,
            "cpu_model": _cpu_model(), "parallel_speedup": speedup, "extrapolated": True,
            "per_shape_1t": per_shape,
            "sample": "one row slab of about %.1f M elements of each of the %d matrix shapes "
                      "(K=%d, r=%d, int%d/%d, %s replicas), steps 2 and 3 of three outer steps "
                      "timed: 1 thread %.1f s; %d threads, one independent slab each, %.1f s; "
                      "per-element rates extrapolated over the %d matrices of the stage"
                      % (target_elems / 1e6, len(shapes), K, r, cfg["qbits"], group,
                         cfg["theta_l"], serial_batch, threads, wall,
                         len(synth.stage_shapes(cfg_id)))}


# ---------------------------------------------------------------------------------------------
# quantise-only outer step
# ---------------------------------------------------------------------------------------------
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
        return None
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
                               "kind": "oracle", "cores_total": os.cpu_count(),
                               "cpu_model": _cpu_model(),
                               "sample": "%d outer steps of one tensor of %d elements (K=%d, "
                                         "int%d/%d), %.2f s per step" %
                                         (nsteps, T["numel"], K, qbits, group, dtc)}
    del tensors
    gc.collect()
    torch.cuda.empty_cache()
    return out


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


def traffic_probe(args):
    """What the memory system gives the fused kernel's mix of streams under the simplest access
    pattern: dlcx_traffic_probe (flat sweep of the same K + K + 2 arrays, same bytes per element,
    no matrix-core work) on one matrix-sized set of arrays per shape of the configuration."""
    import torch

    import paper_2506_21263_amd as dlcx
    import synth

    dlcx.lib()
    torch.cuda.set_device(0)
    dev = "cuda:0"
    cfg = synth.CONFIGS[args.config]
    K = args.workers or cfg["K"]
    dt = torch.bfloat16 if cfg["theta_l"] == "bf16" else torch.float32
    tl_bytes = 2 if cfg["theta_l"] == "bf16" else 4
    bpp = (8 + tl_bytes) * K + 16
    shapes = []
    for sh in cfg["layer_shapes"]:
        if sh not in shapes:
            shapes.append(sh)
    res = []
    for (m, n) in shapes:
        numel = m * n
        theta, v = torch.randn(numel, device=dev), torch.zeros(numel, device=dev)
        ef = [torch.zeros(numel, device=dev) for _ in range(K)]
        tl = [torch.randn(numel, device=dev).to(dt) for _ in range(K)]
        for _ in range(2):
            dlcx.dlcx_traffic_probe(tl, ef, theta, v)
        torch.cuda.synchronize()
        dlcx.dlcx_profile_enable(True)
        for _ in range(args.steps):
            dlcx.dlcx_traffic_probe(tl, ef, theta, v)
        torch.cuda.synchronize()
        ms, cnt = dlcx.dlcx_profile_read()["traffic_probe"]
        dlcx.dlcx_profile_enable(False)
        res.append({"arrays_of": "%dx%d" % (m, n), "ms_per_launch": ms / cnt,
                    "GBps": bpp * numel / (ms / cnt * 1e-3) / 1e9})
        del theta, v, ef, tl
        torch.cuda.empty_cache()
    worst = min(r["GBps"] for r in res)
    print(json.dumps({"metric": "flat sweep of the fused kernel's traffic mix (dlcx_traffic_probe)",
                      "value": worst, "unit": "GB/s", "frac_of_8TBps": worst / HBM_PEAK_GBS,
                      "bytes_per_element": bpp, "K": K, "theta_l": cfg["theta_l"],
                      "per_shape": res}), flush=True)


# ---------------------------------------------------------------------------------------------
# streams restricted to a subset of the compute units (config 4: the outer step and a synthetic
# inner-step load side by side)
# ---------------------------------------------------------------------------------------------
def masked_stream(device, cu_lo, cu_hi, total_cus=256):
    """A HIP stream (default priority) whose kernels may only use compute units cu_lo .. cu_hi-1
    of the mask handed to hipExtStreamCreateWithCUMask, wrapped for torch."""
    import ctypes as C

    import torch

    hip = C.CDLL("libamdhip64.so")
    words = (total_cus + 31) // 32
    mask = (C.c_uint32 * words)()
    for cu in range(cu_lo, cu_hi):
        mask[cu // 32] |= 1 << (cu % 32)
    handle = C.c_void_p()
    rc = hip.hipExtStreamCreateWithCUMask(C.byref(handle), C.c_uint32(words), mask)
    if rc != 0:
        raise RuntimeError("hipExtStreamCreateWithCUMask failed: %d" % rc)
    _MASKED_STREAMS.append((hip, handle))
    return torch.cuda.ExternalStream(handle.value, device=device)


_MASKED_STREAMS = []


def destroy_masked_streams():
    """The streams of masked_stream are this script's to destroy (torch only wraps them): call
    once nothing is queued on them any more and nothing will be."""
    while _MASKED_STREAMS:
        hip, handle = _MASKED_STREAMS.pop()
        hip.hipStreamDestroy(handle)


# ---------------------------------------------------------------------------------------------
# low-rank outer step (the headline)
# ---------------------------------------------------------------------------------------------
def lowrank(args):
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
    adaptive = args.config == 3
    gemm_load = args.gemm_load
    if gemm_load < 0:
        gemm_load = 20 if args.config == 4 else 0
    # config 4: the outer step's streams keep off the compute units reserved for the load
    stream_pool = None
    load_cus = args.load_cus if args.load_cus >= 0 else (64 if args.config == 4 else 0)
    if not gemm_load:
        load_cus = 0
    if load_cus:
        stream_pool = [masked_stream(device, 0, 256 - load_cus) for _ in range(max(args.streams, 1))]
    stage, inputs, gen = build_stage(args.config, args.mma, layers, device, fused, args.streams,
                                     plain=args.probe, workers=args.workers,
                                     iters=args.power_iters, chunk=args.chunk,
                                     requant=args.requant, keep_uv=adaptive,
                                     stream_pool=stream_pool)
    locals_ = [t["theta_l"] for t in inputs]
    if args.probe:
        x = torch.empty(1 << 28, dtype=torch.float32, device=device)
        y = torch.empty_like(x)
        y.copy_(x)  # the plain copy of known size (1 GiB in, 1 GiB out) the counters are scaled by
        for _ in range(2):
            stage.step(locals_)
        torch.cuda.synchronize()
        print("probe done: %d matrices, 2 steps" % len(stage.mats), file=sys.stderr)
        return None
    K = args.workers or cfg["K"]
    params = stage.params()
    selector = RankSelector(stage, c=cfg.get("window", 5), r1=cfg["r"], rmin=cfg.get("rmin", 4),
                            rmax=cfg.get("rmax", cfg["r"]), H1=125)
    selector.first()
    ranks = []
    load = None
    if gemm_load:
        # synthetic inner-step load: bf16 GEMMs 8192^3 on a stream of their own
        load = {"stream": (masked_stream(device, 256 - load_cus, 256) if load_cus
                           else torch.cuda.Stream(device=device)),
                "a": torch.randn(8192, 8192, device=device, dtype=torch.bfloat16),
                "b": torch.randn(8192, 8192, device=device, dtype=torch.bfloat16),
                "c": torch.empty(8192, 8192, device=device, dtype=torch.bfloat16)}
    log("stage: %d matrices, %.3f G params, K=%d, %.1f GB allocated" %
        (len(stage.mats), params / 1e9, K, torch.cuda.memory_allocated() / 1e9))

    use_graph = {"on": False}
    if load is not None:
        # Everything of this run is issued from a stream of torch's own (non-blocking) instead of
        # the null stream: streams created with a compute-unit mask are ordinary blocking streams,
        # and every operation on the null stream (the fork and join events of a step) would wait
        # for, and be waited for by, all work on them -- the load and the step would serialise.
        # The stream it is issued from is the first of the stage's own rather than one more: the
        # process has four hardware queues, and with the three of the stage, the load's and a
        # further one two streams share a queue and wait for each other (4 % on the step).
        torch.cuda.set_stream(stage.side[0] if stage.side else torch.cuda.Stream(device=device))

    def issue_load():
        with torch.cuda.stream(load["stream"]):
            for _ in range(gemm_load):
                torch.matmul(load["a"], load["b"], out=load["c"])

    def one_step(serial=False, with_load=True):
        if use_graph["on"] and not serial:
            stage.replay()
            rp, r_next, _ = selector.next(stage.t + 1)
            ranks.append((rp, r_next))
            return
        if load is not None and with_load:
            load["stream"].wait_stream(torch.cuda.current_stream())
            issue_load()
        stage.step(locals_, serial=serial)
        # Alg. 3: measure r' on this round's averages and apply the window rule; only the
        # adaptive configuration lets the result change the rank of the next compression
        rp, r_next, _ = selector.next(stage.t + 1)
        ranks.append((rp, r_next, stage.mats[0].r))
        if load is not None and with_load:
            torch.cuda.current_stream().wait_stream(load["stream"])

    def timed_steps(n, **kw):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            one_step(**kw)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    per_round = None
    overlap = None
    if adaptive:
        # Alg. 3 drives the rank; every round the replicas are redrawn with a fresh spectrum
        # exponent alpha ~ U[0.5, 2] against the current theta_g, OUTSIDE the timed region; each
        # outer step is timed on its own with events on the issuing stream
        per_round = []
        total_ms = 0.0
        for rnd in range(args.warmup + args.steps):
            alpha = float(0.5 + 1.5 * torch.rand(1, generator=gen).item())
            for M, t in zip(stage.mats, inputs):
                synth.torch_redraw_replicas(t, M.theta_g, alpha)
            torch.cuda.synchronize()
            r_now = stage.mats[0].r
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            t0 = time.perf_counter()
            one_step()
            e1.record()
            torch.cuda.synchronize()
            wall_ms = (time.perf_counter() - t0) * 1e3
            rp, r_next = ranks[-1][0], ranks[-1][1]
            if r_next != r_now:
                fresh = None
                if r_next > r_now:  # cannot happen with r' <= r_t, kept for other bounds
                    fresh = [torch.randn(r_next - r_now, M.n, device=device) for M in stage.mats]
                stage.set_rank(r_next, fresh)
            timed = rnd >= args.warmup
            per_round.append({"round": rnd + 1, "alpha": round(alpha, 3), "rank": r_now,
                              "rprime": rp, "rank_next": r_next, "ms": wall_ms,
                              "ms_events": e0.elapsed_time(e1), "timed": timed})
            if timed:
                total_ms += wall_ms
            log("round %d: alpha %.2f rank %d r' %d -> %d  %.1f ms" %
                (rnd + 1, alpha, r_now, rp, r_next, wall_ms))
        dt_step = total_ms * 1e-3 / args.steps
    else:
        for _ in range(args.warmup):
            one_step()
        torch.cuda.synchronize()
        # fixed ranks and no foreign stream: the steady outer step can be recorded once into a
        # HIP graph (all launches on all streams) and replayed; measured, it changes nothing at
        # the large configurations, the host is not what the step waits for
        if args.graph and load is None and stage.t >= 2:
            stage.capture(locals_)
            use_graph["on"] = True
            one_step()
            torch.cuda.synchronize()
        dt_step = timed_steps(args.steps)
        if load is not None:
            # the same steps without the load, the load without the steps
            t_a = timed_steps(args.steps, with_load=False)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                issue_load()
            torch.cuda.synchronize()
            t_c = (time.perf_counter() - t0) / args.steps
            overlap = {"t_step_alone_ms": t_a * 1e3, "t_load_alone_ms": t_c * 1e3,
                       "t_both_ms": dt_step * 1e3,
                       "sum_ms": (t_a + t_c) * 1e3, "max_ms": max(t_a, t_c) * 1e3,
                       # 1.0: the shorter of the two is fully hidden behind the longer
                       "hidden_frac": (t_a + t_c - dt_step) / min(t_a, t_c),
                       "both_over_max": dt_step / max(t_a, t_c),
                       "load": "%d bf16 GEMMs 8192^3 per outer step (%.1f TFLOP) on a stream of "
                               "their own" % (gemm_load, gemm_load * 2 * 8192.0 ** 3 / 1e12),
                       "cus_reserved_for_load": load_cus,
                       "cus_for_outer_step": 256 - load_cus if load_cus else 256}
    ms_per_step = dt_step * 1e3
    value = params / dt_step

    # per-kernel durations: the same steps again with HIP events around every launch, all on
    # one stream so that a kernel's events bracket that kernel alone
    kernels, roofline, dt_prof = {}, None, None
    tl_bytes = 2 if cfg["theta_l"] == "bf16" else 4
    if True:
        # (adaptive configuration: one such step, at the rank the rounds ended on)
        nprof = 1 if adaptive else args.steps
        dlcx.dlcx_profile_enable(True)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(nprof):
            one_step(serial=True, with_load=False)
        torch.cuda.synchronize()
        dt_prof = (time.perf_counter() - t1) * args.steps / nprof
        prof = dlcx.dlcx_profile_read()
        dlcx.dlcx_profile_enable(False)
        for name, (ms, cnt) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            kernels[name] = {"ms_per_step": ms / nprof, "launches_per_step": cnt / nprof}
        dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
        bpp = algorithmic_bytes_per_param(dom, K, tl_bytes, fused)
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
                        "traffic_source": "profiles/pmc_memory_system_round_kernel_vs_flat_sweep_"
                                          "cfg2.txt, profiles/pmc_hbm_traffic_cfg2.txt (counter "
                                          "runs cannot share a process with the timed run)",
                        "algorithmic_bytes_per_param_per_launch": bpp,
                        "avg_launch_ms": kernels[dom]["ms_per_step"] / launches,
                        "launches_per_step": launches}
            if adaptive:
                roofline["at_rank"] = stage.mats[0].r_prev
            if dom == "round_fused" and args.mma != 0 and not adaptive:
                # matrix-core work of the same kernel: r (reconstruction) + r K (projection)
                # multiply-adds per element, each as 3 (bf16x2) or 6 (bf16x3) bf16 piece products
                pieces = 6 if args.mma == 1 else 3
                useful = 2.0 * cfg["r"] * (1 + K) * params
                sec = kernels[dom]["ms_per_step"] * 1e-3
                roofline["mfma"] = {
                    "useful_TFLOPs": useful / sec / 1e12,
                    "useful_frac_of_peak": useful / sec / 1e12 / 2500.0,
                    "executed_bf16_TFLOPs": useful * pieces / sec / 1e12,
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
                  2: "bf16x2-split MFMA, f32 accumulate",
                  3: "bf16x2-split MFMA, projections above rank 64 as one fp16 MFMA product, "
                     "f32 accumulate"}[args.mma],
        "data": "synthetic",
        "config": {"workload": cfg["name"], "layers": layers, "matrices": len(stage.mats),
                   "params": params, "K": K, "rank": cfg["r"], "qbits": cfg["qbits"],
                   "group": cfg["group"], "theta_l": cfg["theta_l"], "mma": args.mma,
                   "fused": fused, "streams": stage.nstreams, "hip_graph": use_graph["on"],
                   "power_iters": args.power_iters, "requant": bool(args.requant)},
        "roofline": roofline,
        "stage_hbm": {"algorithmic_bytes_per_param": b_alg,
                      "achieved_GBps": b_alg * params / dt_step / 1e9,
                      "frac_of_8TBps": b_alg * params / dt_step / 1e9 / HBM_PEAK_GBS},
        "kernels": kernels,
        "rank_trace": [list(x) for x in ranks[-(2 * args.steps):][:args.steps]],
    }
    if dt_prof is not None:
        out["ms_per_step_serial_with_events"] = dt_prof / args.steps * 1e3
    if per_round is not None:
        out["config"]["timing"] = ("each outer step timed on its own; replicas redrawn with a "
                                   "fresh alpha ~ U[0.5, 2] between steps, outside the timing")
        out["per_round"] = per_round
        out["rank_trace"] = [[p["rprime"], p["rank_next"], p["rank"]] for p in per_round]
        # matrix-core work at each round's own rank: both projections for K workers and one
        # reconstruction, 2 r (2 K + 1) useful flop per element; executed: every product as 3
        # (bf16 x 2) or 6 (bf16 x 3) piece products, the projections above rank 64 as one fp16
        # product in mode 3
        timed = [p for p in per_round if p["timed"]]
        sec = sum(p["ms"] for p in timed) * 1e-3
        pieces = 6 if args.mma == 1 else 3
        useful = sum(2.0 * p["rank"] * (2 * K + 1) * params for p in timed)
        executed = sum(2.0 * p["rank"] * params *
                       (2 * K * (1 if args.mma == 3 and p["rank"] > 64 else pieces) + pieces)
                       for p in timed)
        out["mfma"] = {"useful_TFLOPs": useful / sec / 1e12,
                       "useful_frac_of_peak": useful / sec / 1e12 / 2500.0,
                       "executed_TFLOPs": executed / sec / 1e12,
                       "peak_bf16_fp16_TFLOPs": 2500.0}
    if overlap is not None:
        out["overlap"] = overlap
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, K, cfg["r"], iters=args.power_iters,
                                           requant=args.requant)
    torch.cuda.synchronize()
    # back to torch's default stream before the streams of this run go away
    torch.cuda.set_stream(torch.cuda.default_stream(torch.device(device)))
    del stage, inputs, locals_, load, selector
    gc.collect()
    torch.cuda.empty_cache()
    destroy_masked_streams()
    return out


def other_configs(args):
    """Compact figures of three more workloads under the same clock as the headline: each is
    built, warmed, timed for a few outer steps and freed before the next."""
    res = {}

    def compact(o):
        c = {"workload": o["config"]["workload"], "ms_per_step": o["ms_per_step"],
             "params_per_s": o["value"], "steps": o["steps"], "warmup": o["warmup"]}
        if o.get("stage_hbm"):
            c["stage_frac_of_8TBps"] = o["stage_hbm"]["frac_of_8TBps"]
            c["stage_bytes_per_param"] = o["stage_hbm"]["algorithmic_bytes_per_param"]
        if o.get("roofline"):
            c["dominant_kernel"] = o["roofline"]["kernel"]
            c["dominant_kernel_frac"] = o["roofline"]["frac"]
        if o.get("kernels"):
            c["launches_per_step"] = sum(k["launches_per_step"] for k in o["kernels"].values())
        c["hip_graph"] = o["config"].get("hip_graph", False)
        return c

    a = copy.copy(args)
    a.config, a.steps, a.warmup, a.layers, a.no_cpu_baseline = 1, 10, 3, 0, True
    a.graph, a.workers, a.gemm_load, a.load_cus = False, 0, 0, 0
    res["cfg1"] = compact(lowrank(a))
    q = copy.copy(a)
    q.quant_only = True
    res["cfg1-quant-only"] = compact(quant_only(q))
    g = copy.copy(a)
    g.config, g.steps, g.warmup, g.graph, g.streams = 0, 200, 5, True, 1
    res["cfg0-graph"] = compact(lowrank(g))
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration (synth.CONFIGS)")
    ap.add_argument("--mma", type=int, default=-1,
                    help="0 fma/fp64-acc, 1 fp32-accurate MFMA, 2 bf16 MFMA, 3 bf16 MFMA with fp16 "
                         "projections above rank 64 (default: 3 at config 3, whose ranks are "
                         "above 64, else 2; at ranks up to 64 the two are the same kernels)")
    ap.add_argument("--layers", type=int, default=0, help="layers resident (0 = the whole stage)")
    ap.add_argument("--unfused", action="store_true", help="separate decompress / Nesterov kernels")
    ap.add_argument("--streams", type=int, default=3, help="HIP streams the matrices are dealt to")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="leave out the other_configs block of the default run")
    ap.add_argument("--gemm-load", type=int, default=-1,
                    help="bf16 8192^3 GEMMs issued on a stream of their own per outer step "
                         "(default: 20 at config 4, else 0)")
    ap.add_argument("--load-cus", type=int, default=-1,
                    help="compute units reserved for the GEMM load (the outer step's streams are "
                         "created with a mask that leaves them out; 0 = no masks; default 64 at "
                         "config 4)")
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
    ap.add_argument("--traffic-probe", action="store_true",
                    help="time the flat sweep of the fused kernel's traffic mix and exit")
    ap.add_argument("--probe", action="store_true",
                    help="counter run: plain random inputs, one 1 GiB copy, two steps, no timing")
    args = ap.parse_args()
    if args.mma < 0:
        args.mma = 3 if args.config == 3 else 2
    if args.gpus != 1:
        print("bench.py: this build measures ONE MI355X; --gpus %d is not supported "
              "(no collectives, no second GPU in this run)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.mfma_peak:
        return mfma_peak(args)
    if args.traffic_probe:
        return traffic_probe(args)
    out = quant_only(args) if args.quant_only else lowrank(args)
    if out is None:
        return
    headline = (args.config == 2 and not args.quant_only and not args.layers and not args.workers
                and args.mma == 2 and not args.unfused)
    if headline and not args.no_other_configs:
        out["other_configs"] = other_configs(args)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
