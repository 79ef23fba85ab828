"""GPU parity of whole outer steps (Alg. 2 with the one-step delay) against the oracle.

Both sides run freely from the same seeded inputs for several rounds; nothing computed on the GPU
is ever fed to the oracle (the local replicas of round t are built from the ORACLE's theta).

What is compared.  delta_i, theta_g, v and the decompressed average Delta_hat are unique and are
compared in rel-L2.  A quantised code is an integer decided by a float: the two sides quantise
factors that differ in the last bits, so a value that sits on a rounding boundary may legitimately
land one step apart.  Codes are therefore compared bit for bit, and a mismatch is accepted only
if it is by one step on a value within 1e-2 of a boundary; when any such flip happened the float
bar of that round is widened to the size of the flipped steps (stated in `flip_allowance`).
"""
import numpy as np
import pytest
import torch

import paper_2506_21263_amd as dlcx
import synth
from oracle import pipeline, ref
from paper_2506_21263_amd.stage import MatrixState, Stage
from gpu_util import DEV, code_mismatch_report, rel_l2, to_dev, to_np

pytestmark = pytest.mark.gpu

TOL = {dlcx.MMA_FMA: 1e-5, dlcx.MMA_F32: 1e-5, dlcx.MMA_BF16: 2e-3}
MODES = [dlcx.MMA_FMA, dlcx.MMA_F32, dlcx.MMA_BF16]
MODE_IDS = ["mma_fma", "mma_f32", "mma_bf16"]

CASES = [
    # name, m, n, K, r, qbits, group, theta_l, rounds, sigma
    ("cfg0", 512, 512, 2, 8, 4, 64, "f32", 3, 1e-3),
    ("cfg1-like", 1024, 2048, 4, 32, 4, 128, "f32", 3, 1e-3),
    ("cfg2-like", 1024, 768, 4, 64, 4, 128, "bf16", 2, 1e-3),
    ("cfg4-like", 768, 1024, 8, 64, 8, 64, "bf16", 2, 1e-3),
]


def flip_allowance(n_flips, count, K):
    """rel-L2 a factor mean can move when n_flips of its K*count codes move by one step.
    One step is about 0.4 of the rms of its group for int4 (less for int8): the mean moves by
    step/K on n_flips elements of count."""
    return 0.5 * np.sqrt(n_flips / float(count)) / K


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_outer_rounds_match_oracle(case, mma):
    name, m, n, K, r, qbits, group, kind, T, sigma = case
    inp = synth.MatrixInputs(m, n, K, r, seed=sum(map(ord, name)), sigma=sigma, alpha=1.0,
                             theta_l=kind)
    orc = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, qbits, group, synth.LR, synth.MU)
    M = MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), qbits, group, mma)
    st = Stage([M], synth.LR, synth.MU)
    tol = TOL[mma]
    allow = 0.0  # flips move the state for good (error feedback): the allowance accumulates
    for t in range(1, T + 1):
        tl = [inp.theta_local(orc.theta, t, i) for i in range(K)]
        orc.step(tl)
        st.step([[to_dev(x) for x in tl]])
        torch.cuda.synchronize()
        for tag, codes_gpu, scales_gpu, L in (("P", M.codes_p, M.scales_p, m),
                                              ("Q", M.codes_q, M.scales_q, n)):
            flips = 0
            for k in range(K):
                nb, ok = code_mismatch_report(to_np(codes_gpu[k]), orc.trace[tag + "_codes"][k],
                                              orc.trace[tag][k], orc.trace[tag + "_scales"][k],
                                              r * L, qbits, group, ref.unpack_codes)
                assert ok, (name, t, tag, k, "code mismatch that is not a boundary flip")
                flips += nb
                if mma != dlcx.MMA_BF16:
                    assert rel_l2(to_np(scales_gpu[k]), orc.trace[tag + "_scales"][k]) <= tol
            if mma != dlcx.MMA_BF16:
                # on the fp32 paths flips are rare events
                assert flips <= max(2, 1e-4 * K * r * L), (name, t, tag, flips)
            allow = max(allow, flip_allowance(flips, r * L, K))
        for k in range(K):
            assert rel_l2(to_np(M.ef[k]), orc.trace["delta"][k]) <= tol + allow, (name, t, k)
        d_hat = torch.zeros(m, n, device=DEV)
        dlcx.dlcx_decompress(M.desc(), M.p_hat, M.q_bar, d_hat)
        cond = np.linalg.cond(orc.trace["p_bar"].astype(np.float64))
        bar = (tol + allow) * max(1.0, cond / 50.0) if mma == dlcx.MMA_BF16 else tol + allow
        assert rel_l2(to_np(d_hat), orc.delta_hat()) <= max(bar, 4e-7 * cond), (name, t, cond, allow)
        assert rel_l2(to_np(M.theta_g), orc.theta) <= tol, (name, t)
        assert rel_l2(to_np(M.v), orc.v) <= tol + allow, (name, t)
        # warm start for the next round, on both sides
        orc.set_basis(orc.q_bar)
        M.q_in.copy_(M.q_bar)
    assert st.t == T and orc.n_applied == T - 1


def test_theta_untouched_in_round_one_and_telescoping_on_gpu():
    # one-step delay: nothing is applied at t = 1; and for the GPU's own outputs the error
    # feedback telescopes: sum_t Delta_hat^t + e^{T+1} = sum_t g^t for every worker.
    m, n, K, r = 256, 384, 3, 8
    inp = synth.MatrixInputs(m, n, K, r, seed=77, sigma=1e-3, alpha=1.0)
    M = MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), 4, 64, dlcx.MMA_FMA)
    st = Stage([M], synth.LR, synth.MU)
    sum_g = [np.zeros((m, n)) for _ in range(K)]
    sum_d = np.zeros((m, n))
    theta_host = inp.theta_g.copy()
    T = 4
    for t in range(1, T + 1):
        tl = [inp.theta_local(theta_host, t, i) for i in range(K)]
        theta_before = to_np(M.theta_g).astype(np.float64)
        st.step([[to_dev(x) for x in tl]])
        torch.cuda.synchronize()
        if t == 1:
            assert np.array_equal(to_np(M.theta_g), inp.theta_g)
        for i in range(K):
            sum_g[i] += theta_before - tl[i].astype(np.float64)
        d_hat = torch.zeros(m, n, device=DEV)
        dlcx.dlcx_decompress(M.desc(), M.p_hat, M.q_bar, d_hat)
        sum_d += to_np(d_hat)
        M.q_in.copy_(M.q_bar)
    for i in range(K):
        e_next = to_np(M.ef[i]).astype(np.float64) - to_np(d_hat)
        assert rel_l2(sum_d + e_next, sum_g[i]) <= 1e-6 * T
