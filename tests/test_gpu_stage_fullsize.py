"""The whole stage of the ~100B-class configurations in the launch configuration bench.py times
(as many layers resident as fit, three HIP streams, lane-wise batches, bf16 MFMA mode, fused
round kernel, bf16 local replicas): K = 4, r = 64, int4 / 128 (all ten layers); the same at
r = 256, the first rank of the adaptive configuration; and K = 8, r = 64, int8 / 64.

No oracle can sweep 8.6 G elements, so this file checks what holds at any size: the one-step
delay of Alg. 2 (nothing applied in round 1, something applied in round 2), orthonormal P_hat,
the quantiser's invariants on sampled groups of the payloads, the range of r' -- and that the
three-stream schedule produces, bit for bit, the state the same steps produce when every kernel
is issued on one stream in matrix order (a race between streams, or a workspace shared by two
lanes, would show up here and nowhere else).
"""
import numpy as np
import pytest
import torch

import bench
import paper_2506_21263_amd as dlcx
import synth
from oracle import ref
from gpu_util import DEV, to_np

pytestmark = pytest.mark.gpu

STEPS = 3
# product arithmetic of each configuration, as bench.py times it
MODE = {2: dlcx.MMA_BF16, 3: dlcx.MMA_F16, 4: dlcx.MMA_BF16}


def _digest(t):
    """Three wrap-around sums over the bit patterns of t (all of it and two strided subsets)."""
    x = t.reshape(-1)
    x = x.view(torch.int32) if x.element_size() == 4 else x.view(torch.int16) if x.element_size() == 2 else x
    return torch.stack([x.sum(dtype=torch.int64), x[::7].sum(dtype=torch.int64),
                        x[3::13].sum(dtype=torch.int64)])


def _state_digest(stage):
    out = []
    for M in stage.mats:
        for t in [M.theta_g, M.v, M.p_hat[: M.r], M.q_bar[: M.r]] + M.ef + M.codes_p + M.scales_p + \
                M.codes_q + M.scales_q:
            out.append(_digest(t))
    out.append(_digest(stage.rprime_dev))
    return torch.stack(out).cpu().numpy()


def _input_digest(stage, locals_):
    out = []
    for M, tl in zip(stage.mats, locals_):
        for t in [M.theta_g, M.q_in] + list(tl):
            out.append(_digest(t))
    return torch.stack(out).cpu().numpy()


def _layers_that_fit(cfg):
    per_layer = sum(m * n for m, n in cfg["layer_shapes"]) * (8 + cfg["K"] * 6) * 1.02
    free, _ = torch.cuda.mem_get_info()
    return int(min(cfg["layers"], (free - 6e9) // per_layer))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("CFG", [2, 3, 4])
def test_whole_stage_three_streams_properties_and_single_stream_bits(CFG):
    torch.cuda.empty_cache()
    cfg = synth.CONFIGS[CFG]
    layers = _layers_that_fit(cfg)
    print("whole-stage case: config %d, %d layers resident" % (CFG, layers), flush=True)
    assert layers >= 4, "not enough free device memory for a meaningful stage"
    K, r, G = cfg["K"], cfg["r"], cfg["group"]
    qbits = cfg["qbits"]
    qmax = 2 ** (qbits - 1) - 1

    stage, inputs_, _ = bench.build_stage(CFG, MODE[CFG], layers, DEV, True, 3)
    locals_ = [t["theta_l"] for t in inputs_]
    assert stage.nstreams == 3 and stage.batched and len(stage.mats) == 7 * layers
    inputs = _input_digest(stage, locals_)
    theta0 = torch.stack([_digest(M.theta_g) for M in stage.mats]).cpu().numpy()

    stage.step(locals_)
    torch.cuda.synchronize()
    print("round 1 done", flush=True)
    # Alg. 2: no average exists in the first round, so the outer optimiser applies nothing
    assert np.array_equal(torch.stack([_digest(M.theta_g) for M in stage.mats]).cpu().numpy(), theta0)
    assert not torch.stack([_digest(M.v) for M in stage.mats]).any()
    for _ in range(STEPS - 1):
        stage.step(locals_)
    torch.cuda.synchronize()
    print("round %d done" % STEPS, flush=True)
    theta_n = torch.stack([_digest(M.theta_g) for M in stage.mats]).cpu().numpy()
    assert all((theta_n[a] != theta0[a]).any() for a in range(len(stage.mats)))

    rs = np.random.default_rng(5)
    rprime = stage.rprime_dev.cpu().numpy()
    assert rprime.min() >= 1 and rprime.max() <= r
    for a in range(0, len(stage.mats), 5):
        M = stage.mats[a]
        p = to_np(M.p_hat[: M.r]).astype(np.float64)
        assert np.abs(p @ p.T - np.eye(M.r)).max() <= 1e-5, ("P_hat not orthonormal", a)
        for codes, scales, L in ((M.codes_p, M.scales_p, M.m), (M.codes_q, M.scales_q, M.n)):
            k = int(rs.integers(K))
            c_host, s_host = to_np(codes[k]), to_np(scales[k])
            for g in rs.choice(M.r * L // G, 8, replace=False):
                c = ref.unpack_codes(c_host[g * G * qbits // 8:(g + 1) * G * qbits // 8], G, qbits)
                top = int(np.abs(c).max())
                # the element of largest magnitude gets +-qmax; an all-zero group has scale 0
                assert top == qmax or (top == 0 and s_host[g] == 0.0), (a, k, int(g), top)
                assert np.isfinite(s_host[g]) and s_host[g] >= 0.0
    for a in (0, len(stage.mats) - 1):
        for e in stage.mats[a].ef:
            assert bool(torch.isfinite(e[:64]).all())
    multi = _state_digest(stage)

    del stage, locals_, inputs_, M, e, codes, scales
    torch.cuda.empty_cache()
    stage, inputs_, _ = bench.build_stage(CFG, MODE[CFG], layers, DEV, True, 3)
    locals_ = [t["theta_l"] for t in inputs_]
    assert np.array_equal(_input_digest(stage, locals_), inputs), "the seeded generator did not repeat"
    for _ in range(STEPS):
        stage.step(locals_, serial=True)
    torch.cuda.synchronize()
    print("single-stream rounds done", flush=True)
    single = _state_digest(stage)
    diff = np.nonzero((multi != single).any(axis=1))[0]
    assert diff.size == 0, ("state entries that differ between the schedules", diff[:10])
