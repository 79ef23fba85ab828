"""GPU parity of the quantise-only outer step (Alg. 1 without the low-rank step, Sec. 4.1), of the
re-quantised average and of the error-buffer update, through the C ABI.

This path has no reduction whose order could differ between the two sides (the mean is an fp64
sum of exact products in worker order, rounded once; everything else is one fp32 operation of
the definition), so the bar is bit-exact for every output, floats included, with both sides
running free for several outer steps.
"""
import numpy as np
import pytest
import torch

import paper_2506_21263_amd as dlcx
import synth
from oracle import pipeline, ref
from gpu_util import DEV, to_dev, to_np

pytestmark = pytest.mark.gpu


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def replicas(rng, theta, K, kind):
    """theta_l,i = theta - g_i with a heavy-tailed g (groups see very different magnitudes)."""
    out = []
    for _ in range(K):
        g = 1e-2 * rng.standard_normal(theta.size) * (1.0 + rng.uniform(0, 3, theta.size) ** 4)
        x = (theta.astype(np.float64) - g).astype(np.float32)
        out.append(synth.f32_to_bf16_bits(x) if kind == "bf16" else x)
    return out


def payload(numel, qbits, group, K):
    cb = numel // 2 if qbits == 4 else numel
    codes = [torch.zeros(cb, device=DEV, dtype=torch.uint8) for _ in range(K)]
    scales = [torch.zeros(numel // group, device=DEV, dtype=torch.float32) for _ in range(K)]
    return codes, scales


CASES = [  # qbits, group, K, theta_l kind, requant, groups, payload written in place
    (4, 64, 2, "f32", False, 1037, False),
    (4, 128, 4, "bf16", False, 523, True),
    (8, 64, 3, "bf16", False, 260, True),
    (8, 16, 1, "f32", False, 4099, False),
    (4, 256, 5, "bf16", True, 129, False),
    (4, 32, 4, "f32", True, 2050, True),
    (8, 128, 16, "bf16", True, 67, True),
]


@pytest.mark.parametrize("qbits,group,K,kind,requant,ngroups,inplace", CASES)
def test_quant_round_runs_free_bit_exact(qbits, group, K, kind, requant, ngroups, inplace):
    numel = group * ngroups
    rng = np.random.default_rng(1000 + numel + K)
    theta0 = (0.02 * rng.standard_normal(numel)).astype(np.float32)
    orc = pipeline.TensorOracle(theta0, K, qbits, group, synth.LR, synth.MU, requant=requant)
    theta, v = to_dev(theta0), torch.zeros(numel, device=DEV)
    ef = [torch.zeros(numel, device=DEV) for _ in range(K)]
    cur = payload(numel, qbits, group, K)
    nxt = cur if inplace else payload(numel, qbits, group, K)
    for t in range(1, 5):
        tl = replicas(rng, orc.theta, K, kind)
        orc.step(tl)
        prev = (None, None) if t == 1 else cur
        dlcx.dlcx_quant_round(numel, qbits, group, [to_dev(x) for x in tl], ef, theta, v, synth.LR,
                              synth.MU, prev[0], prev[1], nxt[0], nxt[1], requant=requant)
        torch.cuda.synchronize()
        cur, nxt = nxt, cur
        for i in range(K):
            assert np.array_equal(to_np(cur[0][i]), orc.codes[i]), (t, i)
            assert np.array_equal(bits(to_np(cur[1][i])), bits(orc.scales[i])), (t, i)
            assert np.array_equal(bits(to_np(ef[i])), bits(orc.ef[i])), (t, i)
        assert np.array_equal(bits(to_np(theta)), bits(orc.theta)), t
        assert np.array_equal(bits(to_np(v)), bits(orc.v)), t
    assert orc.n_applied == 3


@pytest.mark.parametrize("qbits,group,K,requant", [(4, 128, 4, False), (8, 64, 3, True)])
def test_separate_entry_points_equal_the_fused_sweep(qbits, group, K, requant):
    # dequant-average (+ re-encoding) -> error buffers -> pseudo-gradients -> OuterOpt ->
    # quantiser, one entry point each, against dlcx_quant_round from the same state.  Payloads and
    # pseudo-gradients must agree bit for bit; dlcx_outer_nesterov evaluates the update with fp32
    # fused multiply-adds instead of fp64, so theta and v agree to an ulp and the separate
    # sequence restarts every round from the fused state.
    numel = group * 331
    rng = np.random.default_rng(77 + K)
    theta0 = (0.02 * rng.standard_normal(numel)).astype(np.float32)
    theta, v = to_dev(theta0), torch.zeros(numel, device=DEV)
    ef = [torch.zeros(numel, device=DEV) for _ in range(K)]
    pay = payload(numel, qbits, group, K)
    d_hat = torch.zeros(numel, device=DEV)
    for t in range(1, 4):
        tl = [to_dev(x) for x in replicas(rng, to_np(theta), K, "bf16")]
        s_theta, s_v = theta.clone(), v.clone()
        s_ef = [e.clone() for e in ef]
        s_pay = ([c.clone() for c in pay[0]], [x.clone() for x in pay[1]])
        prev = (None, None) if t == 1 else pay
        dlcx.dlcx_quant_round(numel, qbits, group, tl, ef, theta, v, synth.LR, synth.MU, prev[0],
                              prev[1], pay[0], pay[1], requant=requant)
        if t >= 2:
            dlcx.dlcx_dequant_average(s_pay[0], s_pay[1], numel, qbits, group, d_hat)
            if requant:
                dlcx.dlcx_requantize(d_hat, numel, qbits, group)
            dlcx.dlcx_ef_update(s_ef, d_hat)
        for i in range(K):
            dlcx.dlcx_delta_ef(s_theta, tl[i], s_ef[i])
        if t >= 2:
            dlcx.dlcx_outer_nesterov(s_theta, s_v, d_hat, synth.LR, synth.MU)
        for i in range(K):
            dlcx.dlcx_quantize(s_ef[i], qbits, group, s_pay[0][i], s_pay[1][i])
        torch.cuda.synchronize()
        for i in range(K):
            assert torch.equal(pay[0][i], s_pay[0][i])
            assert torch.equal(pay[1][i].view(torch.int32), s_pay[1][i].view(torch.int32))
            assert torch.equal(ef[i].view(torch.int32), s_ef[i].view(torch.int32))
        assert torch.allclose(theta, s_theta, rtol=1e-6, atol=5e-8)
        assert torch.allclose(v, s_v, rtol=1e-6, atol=5e-8)
        assert (t == 1) == bool(torch.equal(theta, to_dev(theta0)))


@pytest.mark.parametrize("qbits,group", [(4, 16), (4, 128), (8, 64), (8, 256)])
def test_requantize_bit_exact(qbits, group):
    count = group * 1031
    rng = np.random.default_rng(5 + group)
    x = (rng.standard_normal(count) * np.exp(rng.uniform(-20, 3, count))).astype(np.float32)
    x[:group] = 0.0
    x[group:2 * group] = 1e-40
    want = pipeline.requantize(x, qbits, group)
    got = to_dev(x)
    dlcx.dlcx_requantize(got, count, qbits, group)
    assert np.array_equal(bits(to_np(got)), bits(want))
    dlcx.dlcx_requantize(got, count, qbits, group)      # a fixed point of the quantiser
    assert np.array_equal(bits(to_np(got)), bits(want))


@pytest.mark.parametrize("numel,K", [(0, 2), (3, 1), (4099, 3), ((1 << 18) + 5, 4)])
def test_ef_update_bit_exact(numel, K):
    rng = np.random.default_rng(numel + K)
    d = rng.standard_normal(numel).astype(np.float32)
    es = [rng.standard_normal(numel).astype(np.float32) for _ in range(K)]
    want = []
    for e in es:
        w = e.copy()
        ref.ef_update(w, d)
        want.append(w)
    dev = [to_dev(e) if numel else torch.zeros(0, device=DEV) for e in es]
    dd = to_dev(d) if numel else torch.zeros(0, device=DEV)
    dlcx.dlcx_ef_update(dev, dd, numel=numel)
    for i in range(K):
        assert np.array_equal(bits(to_np(dev[i])), bits(want[i]))


def test_first_step_leaves_the_outer_state_alone():
    # t = 1: no previous payload, theta and v must come back bit for bit (nothing is applied).
    numel, K, group = 64 * 300, 2, 64
    rng = np.random.default_rng(9)
    theta0 = (0.02 * rng.standard_normal(numel)).astype(np.float32)
    theta, v = to_dev(theta0), torch.full((numel,), 3.0, device=DEV)
    ef = [torch.zeros(numel, device=DEV) for _ in range(K)]
    codes, scales = payload(numel, 4, group, K)
    tl = [to_dev(x) for x in replicas(rng, theta0, K, "f32")]
    dlcx.dlcx_quant_round(numel, 4, group, tl, ef, theta, v, synth.LR, synth.MU, None, None,
                          codes, scales)
    assert np.array_equal(bits(to_np(theta)), bits(theta0))
    assert torch.all(v == 3.0)
