"""GPU parity of whole outer steps (Alg. 2 with the one-step delay) against the oracle.

The compressed pipeline is discontinuous: a factor value that sits on a rounding boundary of the
quantiser lands one code apart when the two sides' float arithmetic differs in the last bit, and
from then on the trailing (noise-level) columns of the orthonormal basis, which are determined
only up to a rotation inside a nearly degenerate subspace, may differ macroscopically.  Two kinds
of test follow from that:

* lockstep: the oracle runs the rounds; before every entry-point call the GPU is given the
  ORACLE's inputs of that call and its outputs are compared (floats in rel-L2 at the mode's bar,
  codes bit for bit, a mismatch being accepted only if it is by one step on a value within 1e-2
  of a rounding boundary).  Nothing computed on the GPU is ever fed to the oracle.
* free-running: the library's own call sequence (stage driver) runs the rounds on the GPU and is
  compared with the oracle strictly until the first code flip; after a flip only what stays
  well defined is checked (the flip is by one step on a boundary value, theta_g at a loose bar,
  and the error-feedback telescoping identity of the GPU's own outputs).
"""
import ctypes

import numpy as np
import pytest
import torch

import paper_2506_21263_amd as dlcx
import synth
from oracle import pipeline, ref
from paper_2506_21263_amd.stage import MatrixState, Stage
from gpu_util import (DEV, GUARD, close, code_mismatch_report, payload_buffers, rel_l2, to_dev,
                      to_np, ws_for)

pytestmark = pytest.mark.gpu

TOL = GUARD
MODES = [dlcx.MMA_FMA, dlcx.MMA_F32, dlcx.MMA_BF16]
MODE_IDS = ["mma_fma", "mma_f32", "mma_bf16"]

CASES = [
    # name, m, n, K, r, qbits, group, theta_l, rounds, sigma
    ("cfg0", 512, 512, 2, 8, 4, 64, "f32", 3, 1e-3),
    ("cfg1-like", 1024, 2048, 4, 32, 4, 128, "f32", 3, 1e-3),
    ("cfg2-like", 1024, 768, 4, 64, 4, 128, "bf16", 2, 1e-3),
    ("cfg4-like", 768, 1024, 8, 64, 8, 64, "bf16", 2, 1e-3),
    ("ragged", 528, 336, 3, 20, 4, 16, "bf16", 2, 1e-3),
    # ranks above 64: the fused entry point takes the sweep-plus-projection form
    ("rank96", 640, 2048, 2, 96, 4, 128, "bf16", 2, 1e-3),
    ("rank128-K3", 768, 1280, 3, 128, 4, 128, "bf16", 2, 1e-3),
    ("rank256-K5", 2048, 512, 5, 256, 8, 64, "f32", 2, 1e-3),
    # degenerate sizes: one worker, rank 1, a single quantiser group per row; the most workers
    ("tiny", 16, 32, 1, 1, 4, 16, "f32", 3, 1e-3),
    ("K16", 64, 48, 16, 12, 8, 16, "bf16", 2, 1e-3),
]


def _check_own_codes(name, t, tag, k, codes_gpu, scales_gpu, factor_gpu, qbits, group):
    """The fp16 form of the projections is accurate to a few 1e-4 of a factor, which is up to a
    few hundredths of an int8 step: its codes legitimately differ from the oracle's far from any
    rounding boundary.  What is exact there: the payload is the quantiser of the GPU's OWN factor
    (which is itself within the mode's bar of the oracle's), codes and scales bit for bit."""
    cw, sw = ref.quantize(np.ascontiguousarray(factor_gpu), qbits, group)
    assert np.array_equal(to_np(codes_gpu), cw), (name, t, tag, k)
    assert np.array_equal(to_np(scales_gpu).view(np.uint32), sw.view(np.uint32)), (name, t, tag, k)
    return 0


def _check_codes(name, t, tag, k, codes_gpu, orc, count, qbits, group):
    nb, ok = code_mismatch_report(to_np(codes_gpu), orc.trace[tag + "_codes"][k], orc.trace[tag][k],
                                  orc.trace[tag + "_scales"][k], count, qbits, group,
                                  ref.unpack_codes)
    assert ok, (name, t, tag, k, "code mismatch that is not a one-step boundary flip")
    return nb


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_lockstep_rounds(case, mma):
    name, m, n, K, r, qbits, group, kind, T, sigma = case
    inp = synth.MatrixInputs(m, n, K, r, seed=sum(map(ord, name)), sigma=sigma, alpha=1.0,
                             theta_l=kind)
    orc = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, qbits, group, synth.LR, synth.MU)
    d = dlcx.desc(m, n, r, qbits, group, mma)
    ws = ws_for(d, K)
    tol = TOL[mma]
    total_flips = 0
    for t in range(1, T + 1):
        # the oracle's state at the start of the round
        theta0, v0 = orc.theta.copy(), orc.v.copy()
        ef0 = [e.copy() for e in orc.ef]
        p_prev = None if orc.p_hat is None else orc.p_hat.copy()
        q_prev = None if orc.q_bar is None else orc.q_bar.copy()
        tl = [inp.theta_local(orc.theta, t, i) for i in range(K)]
        orc.step(tl)
        # --- error buffer and outer update from the previous round's average
        efs = [to_dev(e) for e in ef0]
        if t >= 2:
            d_hat = torch.zeros(m, n, device=DEV)
            dlcx.dlcx_decompress(d, to_dev(p_prev), to_dev(q_prev), d_hat, efs, workspace=ws)
            assert close(to_np(d_hat), orc.trace["delta_hat_prev"], tol), (name, t)
            for k in range(K):
                assert close(ef0[k] - to_np(efs[k]), ef0[k] - orc.trace["e"][k], tol)
            efs = [to_dev(e) for e in orc.trace["e"]]
            th, v = to_dev(theta0), to_dev(v0)
            dlcx.dlcx_outer_nesterov(th, v, to_dev(orc.trace["delta_hat_prev"]), synth.LR, synth.MU)
            assert rel_l2(to_np(th), orc.theta) <= 1e-6 and rel_l2(to_np(v), orc.v) <= 1e-6
            # fused form: decompress + error buffers + outer update in one pass
            efs2 = [to_dev(e) for e in ef0]
            th2, v2 = to_dev(theta0), to_dev(v0)
            dlcx.dlcx_decompress_apply(d, to_dev(p_prev), to_dev(q_prev), efs2, th2, v2, synth.LR,
                                       synth.MU, workspace=ws)
            assert close(theta0 - to_np(th2), theta0 - orc.theta, tol), (name, t)
            assert close(to_np(v2), orc.v, tol)
            for k in range(K):
                assert close(ef0[k] - to_np(efs2[k]), ef0[k] - orc.trace["e"][k], tol)
            # fully fused form: error buffers, next pseudo-gradients and outer update in one pass
            efs3 = [to_dev(e) for e in ef0]
            th3, v3 = to_dev(theta0), to_dev(v0)
            dlcx.dlcx_ef_delta_apply(d, to_dev(p_prev), to_dev(q_prev), [to_dev(x) for x in tl], efs3,
                                     th3, v3, synth.LR, synth.MU, workspace=ws)
            assert torch.equal(th3, th2) and torch.equal(v3, v2)
            for k in range(K):
                # delta = g + e with e = delta_prev - delta_hat: compare the part the kernel adds
                base = ref.delta_ef(theta0.reshape(-1), np.ascontiguousarray(tl[k]).reshape(-1),
                                    ef0[k].reshape(-1)).reshape(m, n)
                assert close(base - to_np(efs3[k]), base - orc.trace["delta"][k], tol)
                assert close(to_np(efs3[k]), orc.trace["delta"][k], tol)
        # --- pseudo-gradient with error compensation
        for k in range(K):
            dlcx.dlcx_delta_ef(to_dev(theta0), to_dev(tl[k]), efs[k])
            assert rel_l2(to_np(efs[k]), orc.trace["delta"][k]) <= 1e-6, (name, t, k)
        deltas = [to_dev(x) for x in orc.trace["delta"]]
        # --- P phase
        codes, scales = payload_buffers(d, dlcx.PHASE_P, K)
        dlcx.dlcx_compress_batched(d, dlcx.PHASE_P, deltas, to_dev(orc.trace["q_in"]), codes, scales, ws)
        torch.cuda.synchronize()
        factors = to_np(ws[: K * r * m * 4].view(torch.float32)).reshape(K, r, m)
        for k in range(K):
            assert close(factors[k], orc.trace["P"][k], tol), (name, t, "P", k)
            if mma == dlcx.MMA_F16:
                _check_own_codes(name, t, "P", k, codes[k], scales[k], factors[k], qbits, group)
            else:
                total_flips += _check_codes(name, t, "P", k, codes[k], orc, r * m, qbits, group)
        # --- the same through the single fused call (error buffers, pseudo-gradients, outer
        #     update and P-phase compression in one sweep); r_prev = 0 at t = 1
        efs4 = [to_dev(e) for e in ef0]
        th4, v4 = to_dev(theta0), to_dev(v0)
        codes4, scales4 = payload_buffers(d, dlcx.PHASE_P, K)
        dlcx.dlcx_ef_delta_apply_compress(
            d, r if t >= 2 else 0, None if p_prev is None else to_dev(p_prev),
            None if q_prev is None else to_dev(q_prev), [to_dev(x) for x in tl], efs4, th4, v4,
            synth.LR, synth.MU, to_dev(orc.trace["q_in"]), codes4, scales4, ws)
        torch.cuda.synchronize()
        assert close(to_np(th4), orc.theta, tol) and close(to_np(v4), orc.v, tol)
        factors4 = to_np(ws[: K * r * m * 4].view(torch.float32)).reshape(K, r, m)
        for k in range(K):
            assert close(to_np(efs4[k]), orc.trace["delta"][k], tol), (name, t, k)
            assert close(factors4[k], orc.trace["P"][k], 2 * tol), (name, t, "P fused", k)
            cw, sw = ref.quantize(factors4[k], qbits, group)
            assert np.array_equal(to_np(codes4[k]), cw)
            assert np.array_equal(to_np(scales4[k]).view(np.uint32), sw.view(np.uint32))
        p_hat = torch.zeros(r, m, device=DEV)
        dlcx.dlcx_average(d, dlcx.PHASE_P, [to_dev(c) for c in orc.trace["P_codes"]],
                          [to_dev(s) for s in orc.trace["P_scales"]], p_hat, ws)
        cond = np.linalg.cond(orc.trace["p_bar"].astype(np.float64))
        assert rel_l2(to_np(p_hat), orc.p_hat) <= max(1e-5, 4e-7 * cond), (name, t, cond)
        # --- Q phase
        codes, scales = payload_buffers(d, dlcx.PHASE_Q, K)
        dlcx.dlcx_compress_batched(d, dlcx.PHASE_Q, deltas, to_dev(orc.p_hat), codes, scales, ws)
        torch.cuda.synchronize()
        factors = to_np(ws[: K * r * n * 4].view(torch.float32)).reshape(K, r, n)
        for k in range(K):
            assert close(factors[k], orc.trace["Q"][k], tol), (name, t, "Q", k)
            if mma == dlcx.MMA_F16:
                _check_own_codes(name, t, "Q", k, codes[k], scales[k], factors[k], qbits, group)
            else:
                total_flips += _check_codes(name, t, "Q", k, codes[k], orc, r * n, qbits, group)
        q_bar = torch.zeros(r, n, device=DEV)
        dlcx.dlcx_average(d, dlcx.PHASE_Q, [to_dev(c) for c in orc.trace["Q_codes"]],
                          [to_dev(s) for s in orc.trace["Q_scales"]], q_bar, ws)
        assert rel_l2(to_np(q_bar), orc.q_bar) <= 1e-6, (name, t)
        orc.set_basis(orc.q_bar)
    # identical inputs: boundary flips are rare
    assert total_flips <= max(4, 1e-3 * T * K * r * (m + n)), total_flips


@pytest.mark.parametrize("case", [c for c in CASES if c[4] > 64], ids=[c[0] for c in CASES if c[4] > 64])
def test_lockstep_rounds_fp16_form(case):
    # ranks above 64 with the projections as one fp16 product (the Q phase at any shape, the P
    # phase where the two-role kernel runs): same rounds, same checks, at that mode's bar
    test_lockstep_rounds(case, dlcx.MMA_F16)


@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("case", CASES[:3], ids=[c[0] for c in CASES[:3]])
def test_free_running_stage_driver(case, mma, fused):
    name, m, n, K, r, qbits, group, kind, T, sigma = case
    inp = synth.MatrixInputs(m, n, K, r, seed=sum(map(ord, name)) + 1, sigma=sigma, alpha=1.0,
                             theta_l=kind)
    orc = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, qbits, group, synth.LR, synth.MU)
    M = MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), qbits, group, mma)
    st = Stage([M], synth.LR, synth.MU, fused=fused, warm_start=True, measure_rank=True)
    tol = TOL[mma]
    flipped = False
    sum_g = [np.zeros((m, n)) for _ in range(K)]
    sum_d = np.zeros((m, n))
    for t in range(1, T + 1):
        tl = [inp.theta_local(orc.theta, t, i) for i in range(K)]
        theta_before = to_np(M.theta_g).astype(np.float64)
        orc.step(tl)
        st.step([[to_dev(x) for x in tl]])
        torch.cuda.synchronize()
        for i in range(K):
            sum_g[i] += theta_before - (synth.bf16_bits_to_f32(tl[i]) if kind == "bf16" else tl[i])
        d_hat = torch.zeros(m, n, device=DEV)
        dlcx.dlcx_decompress(M.desc(), M.p_hat, M.q_bar, d_hat, workspace=st.workspace)
        sum_d += to_np(d_hat)
        if t == 1:
            assert np.array_equal(to_np(M.theta_g), inp.theta_g)  # nothing applied at t = 1
        if not flipped:
            for tag, cg, L in (("P", M.codes_p, m), ("Q", M.codes_q, n)):
                for k in range(K):
                    if not flipped:
                        flipped = _check_codes(name, t, tag, k, cg[k], orc, r * L, qbits, group) > 0
        if not flipped:  # strict parity while the two code streams are identical
            for k in range(K):
                assert close(to_np(M.ef[k]), orc.trace["delta"][k], tol), (name, t, k)
            cond = np.linalg.cond(orc.trace["p_bar"].astype(np.float64))
            assert rel_l2(to_np(d_hat), orc.delta_hat()) <= max(tol, 4e-7 * cond), (name, t, cond)
            assert close(to_np(M.theta_g), orc.theta, tol) and close(to_np(M.v), orc.v, tol)
        assert rel_l2(to_np(M.theta_g), orc.theta) <= 2e-2, (name, t)  # sanity bar after a flip
        orc.set_basis(orc.q_bar)
    assert st.t == T and orc.n_applied == T - 1
    if not flipped:
        assert int(st.rprime_dev[0].item()) == ref.effective_rank(orc.q_bar, 0.99)
    # error feedback telescopes on the GPU's own outputs, flips or not
    for i in range(K):
        e_next = to_np(M.ef[i]).astype(np.float64) - to_np(d_hat)
        assert rel_l2(sum_d + e_next, sum_g[i]) <= 1e-6 * T


def test_multi_stream_stage_equals_single_stream():
    # dealing the matrices of a stage to several HIP streams changes nothing: bitwise-equal state
    shapes = [(256, 384), (512, 256), (384, 640), (256, 256), (640, 384)]
    K, r = 3, 16

    def run(streams, batched=True, chunk=0):
        mats, tls = [], []
        for a, (m, n) in enumerate(shapes):
            inp = synth.MatrixInputs(m, n, K, r, seed=500 + a, sigma=1e-3, alpha=1.0, theta_l="bf16")
            mats.append(MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), 4, 64, dlcx.MMA_BF16))
            tls.append([to_dev(inp.theta_local(inp.theta_g, 1, i)) for i in range(K)])
        st = Stage(mats, synth.LR, synth.MU, fused=True, warm_start=True, streams=streams,
                   measure_rank=True, batched=batched, chunk=chunk)
        for _ in range(3):
            st.step(tls)
        torch.cuda.synchronize()
        return st

    one, three, loose, chunked = run(1), run(3), run(2, batched=False), run(2, chunk=2)
    assert three.nstreams == 3 and max(len(c) for c in chunked.lane_chunks) >= 2
    for st in (one, three, chunked):   # every matrix in exactly one chunk
        covered = sorted(a for chunks in st.lane_chunks for lo, hi in chunks for a in range(lo, hi))
        assert covered == list(range(len(shapes)))
    for other in (three, loose, chunked):
        for A, B in zip(one.mats, other.mats):
            assert torch.equal(A.theta_g, B.theta_g) and torch.equal(A.v, B.v)
            assert torch.equal(A.q_bar, B.q_bar) and torch.equal(A.p_hat, B.p_hat)
            for x, y in zip(A.ef, B.ef):
                assert torch.equal(x, y)
        assert torch.equal(one.rprime_dev, other.rprime_dev)


def test_adaptive_rank_rounds_config3_like():
    # Alg. 3 end to end on a small stage: 3 matrices, r_1 = 32, window c = 3, bounds [4, 32],
    # spectra that decay faster every round, so the measured r' and with it the rank shrink and
    # every width of the MFMA tiles is exercised.  The GPU is re-seeded with the oracle's state
    # at the start of each round (lockstep at round granularity); r', r_t and H_t are integers
    # and must agree exactly.
    shapes = [(256, 384), (384, 256), (512, 512)]
    K, r1, c, rmin, H1, qbits, group = 2, 32, 3, 4, 125, 4, 64
    T = 7
    alphas = [0.5, 0.75, 1.0, 1.5, 2.0, 2.5, 3.0]
    inps = [synth.MatrixInputs(m, n, K, r1, seed=900 + a, sigma=2e-4, alpha=1.0, theta_l="bf16")
            for a, (m, n) in enumerate(shapes)]
    orcs = [pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, qbits, group, synth.LR, synth.MU)
            for inp in inps]
    hist_o = [r1]
    hist_g = (ctypes.c_int32 * c)()
    rp, r_t, H = dlcx.dlcx_select_rank_from(None, 0, hist_g, 1, c, r1, rmin, r1, H1, rprime=r1)
    assert (r_t, H) == ref.adagradcmp(hist_o, 1, c, r1, rmin, r1, H1)
    r_now = r1
    for t in range(1, T + 1):
        mats, tls = [], []
        for inp, orc in zip(inps, orcs):
            M = MatrixState(to_dev(orc.theta), K, to_dev(orc.q_in), qbits, group, dlcx.MMA_BF16,
                            r_max=r1)
            M.v.copy_(to_dev(orc.v))
            for k in range(K):
                M.ef[k].copy_(to_dev(orc.ef[k]))
            if orc.p_hat is not None:
                M.r_prev = orc.p_hat.shape[0]
                M.p_hat.view(-1)[: orc.p_hat.size].copy_(to_dev(orc.p_hat).view(-1))
                M.q_bar.view(-1)[: orc.q_bar.size].copy_(to_dev(orc.q_bar).view(-1))
            mats.append(M)
            tls.append([inp.theta_local(orc.theta, t, i, alpha=alphas[t - 1]) for i in range(K)])
        st = Stage(mats, synth.LR, synth.MU, fused=True, warm_start=False, measure_rank=True)
        st.t = t - 1
        for orc, tl in zip(orcs, tls):
            orc.step(tl)
        st.step([[to_dev(x) for x in tl] for tl in tls])
        torch.cuda.synchronize()
        for M, orc in zip(mats, orcs):
            assert M.r == r_now and orc.q_bar.shape[0] == r_now
            assert rel_l2(to_np(M.theta_g), orc.theta) <= 2e-3
            for k in range(K):
                assert rel_l2(to_np(M.ef[k]), orc.trace["delta"][k]) <= 2e-3
        # r' per matrix on each side's own average, then the stage value and the window rule
        want_rp = [ref.effective_rank(orc.q_bar, 0.99) for orc in orcs]
        got_rp = to_np(st.rprime_dev).tolist()
        # the GPU's Q_bar differs from the oracle's after code flips: re-measure on the oracle's
        ws = torch.empty(dlcx.dlcx_batched_workspace_bytes([M.desc() for M in mats]), device=DEV,
                         dtype=torch.uint8)
        out = torch.zeros(len(mats), device=DEV, dtype=torch.int32)
        dlcx.dlcx_effective_rank_batched([M.desc() for M in mats],
                                         [to_dev(orc.q_bar) for orc in orcs], 0.99, out, ws)
        assert to_np(out).tolist() == want_rp, (t, got_rp, want_rp)
        hist_o.append(pipeline.stage_rprime(want_rp, rmin))
        want_r, want_H = ref.adagradcmp(hist_o, t + 1, c, r1, rmin, r1, H1)
        rp, r_next, H_next = dlcx.dlcx_select_rank_from(out, len(mats), hist_g, t + 1, c, r1, rmin,
                                                        r1, H1)
        assert (rp, r_next, H_next) == (hist_o[-1], want_r, want_H), t
        # next round's basis: warm start, resized to the new rank, on the oracle side
        for inp, orc in zip(inps, orcs):
            fresh = inp.fresh_basis_columns(t, max(0, r_next - r_now))
            orc.set_basis(pipeline.next_basis(orc.q_bar, r_next, fresh))
        r_now = r_next
    assert r_now < r1, "the rank was expected to shrink with the steeper spectra"


@pytest.mark.parametrize("batched", [True, False])
def test_requantised_factor_averages(batched):
    # Averaged factors re-encoded to q bits before use (what a reduction carrying q-bit values
    # would deliver).  The GPU's own payloads are decoded, averaged and re-encoded by the oracle:
    # Q_bar must match bit for bit, P_hat (orthonormalised afterwards) to the fp32 bar.  Two
    # rounds, so that the re-encoded factors also pass through the fused feedback sweep.
    shapes = [(256, 384), (512, 256)]
    K, r, qbits, group = 3, 8, 4, 64
    mats, tls = [], []
    for a, (m, n) in enumerate(shapes):
        inp = synth.MatrixInputs(m, n, K, r, seed=900 + a, sigma=1e-3, alpha=1.0, theta_l="bf16")
        mats.append(MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), qbits, group, dlcx.MMA_F32))
        tls.append([to_dev(inp.theta_local(inp.theta_g, 1, i)) for i in range(K)])
    st = Stage(mats, synth.LR, synth.MU, fused=True, warm_start=True, streams=2, batched=batched,
               requant=True)
    plain = Stage([MatrixState(M.theta_g.clone(), K, M.q_in[:r].clone(), qbits, group, dlcx.MMA_F32)
                   for M in mats], synth.LR, synth.MU, fused=True, warm_start=True, batched=batched)
    for t in range(2):
        st.step(tls)
        torch.cuda.synchronize()
        for M in mats:
            cp, sp = [to_np(c) for c in M.codes_p], [to_np(s) for s in M.scales_p]
            p_bar = ref.dequant_average(cp, sp, r * M.m, qbits, group)
            p_hat = ref.orthonormalize(pipeline.requantize(p_bar, qbits, group).reshape(r, M.m))
            assert rel_l2(to_np(M.p_hat)[:r], p_hat) <= 1e-5
            cq, sq = [to_np(c) for c in M.codes_q], [to_np(s) for s in M.scales_q]
            q_bar = pipeline.requantize(ref.dequant_average(cq, sq, r * M.n, qbits, group),
                                        qbits, group).reshape(r, M.n)
            assert np.array_equal(to_np(M.q_bar)[:r].view(np.uint32), q_bar.view(np.uint32))
    plain.step(tls)
    torch.cuda.synchronize()
    assert not torch.equal(plain.mats[0].q_bar, mats[0].q_bar)   # the option does something


def test_graph_replay_equals_eager_steps():
    # One outer step recorded into a HIP graph (all launches, all streams) and replayed: the
    # state after every replay must equal, bit for bit, the state of a twin stage stepped
    # eagerly, with eager work of the same library and synchronisations between the replays.
    shapes = [(256, 384), (512, 256), (384, 640), (256, 256)]
    K, r = 3, 16

    def make(streams):
        mats, tls = [], []
        for a, (m, n) in enumerate(shapes):
            inp = synth.MatrixInputs(m, n, K, r, seed=700 + a, sigma=1e-3, alpha=1.0, theta_l="bf16")
            mats.append(MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), 4, 64, dlcx.MMA_BF16))
            tls.append([to_dev(inp.theta_local(inp.theta_g, 1, i)) for i in range(K)])
        return Stage(mats, synth.LR, synth.MU, fused=True, warm_start=True, streams=streams,
                     measure_rank=True), tls

    eager, tls_e = make(3)
    graphed, tls_g = make(3)
    for _ in range(2):
        eager.step(tls_e)
        graphed.step(tls_g)
    torch.cuda.synchronize()
    graphed.capture(tls_g)
    scratch = torch.zeros(1 << 16, device=DEV)
    for rep in range(4):
        eager.step(tls_e)
        graphed.replay()
        torch.cuda.synchronize()
        for A, B in zip(eager.mats, graphed.mats):
            assert torch.equal(A.theta_g, B.theta_g) and torch.equal(A.v, B.v), rep
            assert torch.equal(A.q_bar, B.q_bar) and torch.equal(A.p_hat, B.p_hat), rep
            for x, y in zip(A.ef, B.ef):
                assert torch.equal(x, y), rep
        assert torch.equal(eager.rprime_dev, graphed.rprime_dev), rep
        # eager work between the replays
        dlcx.dlcx_outer_nesterov(scratch, scratch.clone(), scratch.clone(), 0.5, 0.5)
        torch.cuda.synchronize()
    assert eager.t == graphed.t == 6


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
def test_zero_pseudo_gradient_stays_zero(mma, fused):
    # Replicas that did not move (theta_l = theta_g, zero error buffers): every factor, payload
    # and average is exactly zero (no NaN from the orthonormalisation of a zero matrix), theta
    # and v do not change over three outer steps, and the measured r' is 0 (counted as rmin).
    m, n, K, r = 256, 384, 3, 8
    rng = np.random.default_rng(3)
    theta0 = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
    q_in = rng.standard_normal((r, n)).astype(np.float32)
    M = MatrixState(to_dev(theta0), K, to_dev(q_in), 4, 64, mma)
    st = Stage([M], synth.LR, synth.MU, fused=fused, warm_start=False, measure_rank=True)
    tl = [[to_dev(theta0) for _ in range(K)]]
    for _ in range(3):
        st.step(tl)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(M.theta_g), theta0)
    assert not torch.any(M.v != 0) and not torch.any(M.q_bar[:r] != 0)
    assert not torch.any(M.p_hat[:r] != 0)
    for k in range(K):
        assert not torch.any(M.ef[k] != 0)
        assert not torch.any(M.codes_p[k] != 0) and not torch.any(M.codes_q[k] != 0)
    assert int(st.rprime_dev[0]) == 0


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
def test_rank_one_single_worker_lockstep(mma):
    # the smallest compressor: r = 1, K = 1 (the mean is the decoded payload itself).  One round
    # from the oracle's state, every float at the mode's bar, codes against the oracle's
    # quantiser of the GPU's own factor.
    m, n, r, K, qbits, group = 272, 208, 1, 1, 8, 16
    inp = synth.MatrixInputs(m, n, K, r, seed=41, sigma=1e-3, alpha=1.0, theta_l="bf16")
    orc = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, qbits, group, synth.LR, synth.MU)
    M = MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), qbits, group, mma)
    st = Stage([M], synth.LR, synth.MU, fused=True, warm_start=True)
    tol = TOL[mma]
    for t in (1, 2):
        tl = [inp.theta_local(orc.theta, t, 0)]
        # lockstep: the GPU starts the round from the oracle's state
        M.theta_g.copy_(to_dev(orc.theta))
        M.v.copy_(to_dev(orc.v))
        M.ef[0].copy_(to_dev(orc.ef[0]))
        if t == 2:
            M.p_hat[:r].copy_(to_dev(orc.p_hat))
            M.q_bar[:r].copy_(to_dev(orc.q_bar))
        orc.step(tl)
        orc.set_basis(orc.q_bar)
        st.step([[to_dev(tl[0])]])
        torch.cuda.synchronize()
        assert close(to_np(M.ef[0]), orc.trace["delta"][0], tol)
        assert close(to_np(M.theta_g), orc.theta, tol)
        # sign and scale of a rank-one basis are fixed by the positive-diagonal rule
        assert rel_l2(to_np(M.p_hat)[:r], orc.p_hat) <= 20 * tol
        assert rel_l2(to_np(M.q_bar)[:r], orc.q_bar) <= 20 * tol


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
@pytest.mark.parametrize("qbits,K", [(8, 3), (4, 2)])
def test_exactly_representable_input_passes_the_compressor_unchanged(mma, fused, qbits, K):
    # Closed form with the quantiser ON (see the oracle pin of the same name): +-1 factor
    # vectors and singular values qmax * 2^-c make every factor entry +-qmax times a power of
    # two, so the codes are all +-qmax, Delta equals the pseudo-gradient and the second outer
    # step is the Nesterov step of exactly that gradient.  Holds in every product mode: the
    # operands have few enough bits for the bf16 splits to be exact.
    qmax = 2 ** (qbits - 1) - 1
    m, n, r, theta0, tl, q_in, delta = synth.exact_lowrank_case(qmax, K)
    M = MatrixState(to_dev(theta0), K, to_dev(q_in), qbits, 16, mma)
    st = Stage([M], 0.5, 0.0, fused=fused, warm_start=True)
    st.step([[to_dev(x) for x in tl]])
    d_hat = torch.zeros(m, n, device=DEV)
    dlcx.dlcx_decompress(M.desc(), M.p_hat, M.q_bar, d_hat, workspace=st.workspace)
    torch.cuda.synchronize()
    for k in range(K):
        assert np.array_equal(to_np(M.ef[k]), delta)
        codes = ref.unpack_codes(to_np(M.codes_p[k]), r * m, qbits)
        assert np.all(np.abs(codes) == qmax)
        codes = ref.unpack_codes(to_np(M.codes_q[k]), r * n, qbits)
        assert np.all(np.abs(codes) == qmax)
    assert np.max(np.abs(np.abs(to_np(M.p_hat)[:r]) - 0.25)) <= 1e-7
    assert rel_l2(to_np(d_hat), delta) <= 1e-6
    st.step([[to_dev(theta0) for _ in range(K)]])
    torch.cuda.synchronize()
    assert rel_l2(to_np(M.theta_g), -0.5 * delta) <= 1e-6
    assert np.max(np.abs(to_np(M.ef[0]))) <= 1e-6 * np.max(np.abs(delta))


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("batched", [True, False], ids=["batched", "per-matrix"])
def test_further_power_iterations_within_a_round(mma, batched):
    # iters = 3: after the round's first P and Q phase, two more of each on the same
    # pseudo-gradients, every P phase from the Q average just formed.  Lockstep for the later
    # iterations (the GPU projects the oracle's pseudo-gradients on the oracle's basis of that
    # iteration), then the stage driver free-running against the oracle until the first code flip.
    # The later iterations project on a basis that is nearly aligned with the singular vectors,
    # so the sums cancel more and a float error of a few 1e-5 of a group's range is ordinary:
    # the codes are therefore checked against the oracle's quantiser applied to the GPU's own
    # factor (bit for bit), the factor against the oracle's at the mode's bar.
    name, m, n, K, r, qbits, group, kind, iters = "iters3", 528, 400, 3, 12, 8, 16, "bf16", 3
    tol = TOL[mma]
    inp = synth.MatrixInputs(m, n, K, r, seed=97, sigma=1e-3, alpha=1.0, theta_l=kind)
    orc = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, qbits, group, synth.LR, synth.MU,
                                iters=iters)
    M = MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), qbits, group, mma)
    st = Stage([M], synth.LR, synth.MU, fused=True, warm_start=True, measure_rank=True,
               batched=batched, iters=iters)
    d = M.desc()
    ws = ws_for(d, K)
    flipped = False
    for t in (1, 2):
        tl = [inp.theta_local(orc.theta, t, i) for i in range(K)]
        orc.step(tl)
        deltas = [to_dev(x) for x in orc.trace["delta"]]
        for j in range(1, iters):
            sfx = "@%d" % j
            assert np.array_equal(orc.trace["q_in" + sfx], orc.trace["q_bar" + ("@%d" % (j - 1) if j > 1 else "")])
            codes, scales = payload_buffers(d, dlcx.PHASE_P, K)
            dlcx.dlcx_compress_batched(d, dlcx.PHASE_P, deltas, to_dev(orc.trace["q_in" + sfx]),
                                       codes, scales, ws)
            torch.cuda.synchronize()
            factors = to_np(ws[: K * r * m * 4].view(torch.float32)).reshape(K, r, m)
            for k in range(K):
                assert close(factors[k], orc.trace["P" + sfx][k], tol), (t, j, k)
                cw, sw = ref.quantize(factors[k], qbits, group)
                assert np.array_equal(to_np(codes[k]), cw), (t, j, k)
                assert np.array_equal(to_np(scales[k]).view(np.uint32), sw.view(np.uint32))
            p_hat = torch.zeros(r, m, device=DEV)
            dlcx.dlcx_average(d, dlcx.PHASE_P, [to_dev(c) for c in orc.trace["P" + sfx + "_codes"]],
                              [to_dev(s) for s in orc.trace["P" + sfx + "_scales"]], p_hat, ws)
            cond = np.linalg.cond(orc.trace["p_bar" + sfx].astype(np.float64))
            assert rel_l2(to_np(p_hat), orc.trace["p_hat" + sfx]) <= max(1e-5, 4e-7 * cond), (t, j)
            codes, scales = payload_buffers(d, dlcx.PHASE_Q, K)
            dlcx.dlcx_compress_batched(d, dlcx.PHASE_Q, deltas, to_dev(orc.trace["p_hat" + sfx]),
                                       codes, scales, ws)
            torch.cuda.synchronize()
            factors = to_np(ws[: K * r * n * 4].view(torch.float32)).reshape(K, r, n)
            for k in range(K):
                assert close(factors[k], orc.trace["Q" + sfx][k], tol), (t, j, k)
                cw, sw = ref.quantize(factors[k], qbits, group)
                assert np.array_equal(to_np(codes[k]), cw), (t, j, k)
                assert np.array_equal(to_np(scales[k]).view(np.uint32), sw.view(np.uint32))
        # ---- the stage driver, free-running
        st.step([[to_dev(x) for x in tl]])
        torch.cuda.synchronize()
        last = "@%d" % (iters - 1)
        for tag, cg in (("P" + last, M.codes_p), ("Q" + last, M.codes_q)):
            for k in range(K):
                flipped = flipped or not np.array_equal(to_np(cg[k]), orc.trace[tag + "_codes"][k])
        if not flipped:
            cond = np.linalg.cond(orc.trace["p_bar" + last].astype(np.float64))
            d_hat = torch.zeros(m, n, device=DEV)
            dlcx.dlcx_decompress(d, M.p_hat, M.q_bar, d_hat, workspace=st.workspace)
            assert rel_l2(to_np(d_hat), orc.delta_hat()) <= max(tol, 4e-7 * cond), (t, cond)
            assert close(to_np(M.theta_g), orc.theta, tol) and close(to_np(M.v), orc.v, tol)
            for k in range(K):
                assert close(to_np(M.ef[k]), orc.trace["delta"][k], tol), (t, k)
        assert rel_l2(to_np(M.theta_g), orc.theta) <= 2e-2
        # flips or not: the driver's own state is consistent with its own payloads, and it fits
        # the mean pseudo-gradient about as well as the oracle's three iterations do
        cq, sq = [to_np(c) for c in M.codes_q], [to_np(x) for x in M.scales_q]
        assert np.array_equal(to_np(M.q_bar)[:r].reshape(-1).view(np.uint32),
                              ref.dequant_average(cq, sq, r * n, qbits, group).view(np.uint32))
        mean = np.mean([x.astype(np.float64) for x in orc.trace["delta"]], axis=0)
        d_hat = torch.zeros(m, n, device=DEV)
        dlcx.dlcx_decompress(d, M.p_hat, M.q_bar, d_hat, workspace=st.workspace)
        if t == 1:  # identical pseudo-gradients on both sides in the first round
            assert abs(np.linalg.norm(mean - to_np(d_hat)) / np.linalg.norm(mean - orc.delta_hat())
                       - 1) < 1e-2
        orc.set_basis(orc.q_bar)
    if not flipped:
        assert int(st.rprime_dev[0].item()) == ref.effective_rank(orc.q_bar, 0.99)
    # the further iterations fit the mean pseudo-gradient better than the first one did
    mean = np.mean([x.astype(np.float64) for x in orc.trace["delta"]], axis=0)
    first = ref.reconstruct(orc.trace["p_hat"], orc.trace["q_bar"])
    assert np.linalg.norm(mean - orc.delta_hat()) < np.linalg.norm(mean - first)


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
def test_free_running_across_rank_changes(mma, fused):
    """The stage driver carries ITS OWN state over five outer steps whose rank goes
    128 -> 48 -> 96 -> 96 -> 20 (Stage.set_rank: one shrink across 64, one grow across 64, one
    step at an unchanged rank, one more shrink), so every step after the first feeds back and
    applies an average formed at another rank than the one it compresses at -- in the fused call
    both the one-sweep kernel with more previous-rank steps than its own (48 after 128, 20 after
    96) and the sweep-plus-projection form (96 after 48).  Compared with the oracle plus
    pipeline.next_basis strictly until the first code flip, then on what stays well defined."""
    m, n, K, qbits, group, kind = 640, 768, 2, 4, 128, "bf16"
    ranks = [128, 48, 96, 96, 20]
    r_max = max(ranks)
    inp = synth.MatrixInputs(m, n, K, ranks[0], seed=4242, sigma=1e-3, alpha=1.0, theta_l=kind)
    orc = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, qbits, group, synth.LR, synth.MU)
    M = MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), qbits, group, mma, r_max=r_max)
    st = Stage([M], synth.LR, synth.MU, fused=fused, warm_start=True, measure_rank=True)
    tol = TOL[mma]
    flipped = False
    sum_g = [np.zeros((m, n)) for _ in range(K)]
    sum_d = np.zeros((m, n))
    for t, r in enumerate(ranks, start=1):
        assert M.r == r and orc.q_in.shape[0] == r
        tl = [inp.theta_local(orc.theta, t, i) for i in range(K)]
        theta_before = to_np(M.theta_g).astype(np.float64)
        orc.step(tl)
        st.step([[to_dev(x) for x in tl]])
        torch.cuda.synchronize()
        assert M.r_prev == r
        for i in range(K):
            sum_g[i] += theta_before - synth.bf16_bits_to_f32(tl[i])
        d_hat = torch.zeros(m, n, device=DEV)
        dlcx.dlcx_decompress(M.desc(), M.p_hat, M.q_bar, d_hat, workspace=st.workspace)
        sum_d += to_np(d_hat)
        if not flipped:
            for tag, cg, L in (("P", M.codes_p, m), ("Q", M.codes_q, n)):
                for k in range(K):
                    if not flipped:
                        cb = r * L // 2
                        flipped = _check_codes("rank-change", t, tag, k, cg[k][:cb], orc, r * L,
                                               qbits, group) > 0
        if not flipped:
            for k in range(K):
                assert close(to_np(M.ef[k]), orc.trace["delta"][k], tol), (t, r, k)
            cond = np.linalg.cond(orc.trace["p_bar"].astype(np.float64))
            assert rel_l2(to_np(d_hat), orc.delta_hat()) <= max(tol, 4e-7 * cond), (t, r, cond)
            assert close(to_np(M.theta_g), orc.theta, tol) and close(to_np(M.v), orc.v, tol), (t, r)
            assert int(st.rprime_dev[0].item()) == ref.effective_rank(orc.q_bar, 0.99), (t, r)
        # sanity bar after a flip: the two sides may then project the noise part of the mean
        # pseudo-gradient (elementwise std sigma / sqrt(K) against 0.02 for theta: 3.5 % of it
        # per round, most of a rank-96 basis being noise-level directions) on different
        # directions, and theta moves by lr (1 + mu) times that every round
        assert rel_l2(to_np(M.theta_g), orc.theta) <= 1e-1, (t, r)
        if t < len(ranks):
            r_next = ranks[t]
            fresh = inp.fresh_basis_columns(t, max(0, r_next - r))
            orc.set_basis(pipeline.next_basis(orc.q_bar, r_next, fresh))
            st.set_rank(r_next, [to_dev(fresh) if r_next > r else None])
            if not flipped:   # the resized warm start is the oracle's, bit for bit where kept
                torch.cuda.synchronize()
                assert close(to_np(M.q_bar[:r_next]), orc.q_in, tol), (t, r_next)
                if r_next > r:
                    assert np.array_equal(to_np(M.q_bar[r:r_next]), fresh[: r_next - r])
    assert st.t == len(ranks) and orc.n_applied == len(ranks) - 1
    # the error feedback telescopes on the GPU's own outputs across the rank changes
    for i in range(K):
        e_next = to_np(M.ef[i]).astype(np.float64) - to_np(d_hat)
        assert rel_l2(sum_d + e_next, sum_g[i]) <= 1e-6 * len(ranks)


@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
def test_resume_two_plus_one_equals_three_rounds(fused):
    """Checkpoint / resume: the whole outer state is caller-owned -- theta_g, v, the K error
    buffers, the last factors P_hat / Q_bar (Q_bar is also the warm start), their rank and the
    round counter.  Three outer steps in one go against two steps, the state copied to the host
    and into brand-new device buffers behind a new stage driver, then the third step: every
    buffer bit for bit the same."""
    shapes = [(384, 512), (512, 256)]
    K, r, qbits, group = 3, 24, 4, 64
    inps = [synth.MatrixInputs(m, n, K, r, seed=7700 + a, sigma=1e-3, alpha=1.0, theta_l="bf16")
            for a, (m, n) in enumerate(shapes)]

    def fresh_stage(states=None, t=0):
        mats = []
        for a, inp in enumerate(inps):
            M = MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), qbits, group, dlcx.MMA_BF16)
            if states is not None:
                s = states[a]
                M.theta_g.copy_(to_dev(s["theta_g"]))
                M.v.copy_(to_dev(s["v"]))
                for k in range(K):
                    M.ef[k].copy_(to_dev(s["ef"][k]))
                M.p_hat.copy_(to_dev(s["p_hat"]))
                M.q_bar.copy_(to_dev(s["q_bar"]))
                M.r, M.r_prev = s["r"], s["r_prev"]
            mats.append(M)
        st = Stage(mats, synth.LR, synth.MU, fused=fused, warm_start=True, streams=2,
                   measure_rank=True)
        st.t = t
        return st

    def locals_for(st, t):
        # replicas depend on the round only (not on the state), so both runs see the same bytes
        return [[to_dev(inp.theta_local(inp.theta_g, t, i)) for i in range(K)] for inp in inps]

    def snapshot(st):
        torch.cuda.synchronize()
        return [dict(theta_g=to_np(M.theta_g), v=to_np(M.v), ef=[to_np(e) for e in M.ef],
                     p_hat=to_np(M.p_hat), q_bar=to_np(M.q_bar), r=M.r, r_prev=M.r_prev)
                for M in st.mats]

    straight = fresh_stage()
    for t in (1, 2, 3):
        straight.step(locals_for(straight, t))
    want = snapshot(straight)
    first = fresh_stage()
    for t in (1, 2):
        first.step(locals_for(first, t))
    saved = snapshot(first)
    saved_t = first.t
    del first
    resumed = fresh_stage(saved, saved_t)
    resumed.step(locals_for(resumed, 3))
    got = snapshot(resumed)
    assert resumed.t == 3
    for a in range(len(shapes)):
        for key in ("theta_g", "v", "p_hat", "q_bar"):
            assert np.array_equal(got[a][key].view(np.uint32), want[a][key].view(np.uint32)), (a, key)
        for k in range(K):
            assert np.array_equal(got[a]["ef"][k].view(np.uint32), want[a]["ef"][k].view(np.uint32))
        assert (got[a]["r"], got[a]["r_prev"]) == (want[a]["r"], want[a]["r_prev"])
    assert torch.equal(resumed.rprime_dev, straight.rprime_dev)


def test_step_beside_a_foreign_busy_stream_is_bit_equal():
    """The one-step-delay scheme runs the outer step while local training keeps the GPU busy
    (Sec. 2.3).  Outer steps issued while another stream runs a queue of bf16 GEMMs (the
    stand-in for the inner steps) leave, bit for bit, the state they leave when run alone."""
    shapes = [(512, 768), (768, 512), (1024, 256)]
    K, r = 4, 32

    def run(busy):
        mats, tls = [], []
        for a, (m, n) in enumerate(shapes):
            inp = synth.MatrixInputs(m, n, K, r, seed=8800 + a, sigma=1e-3, alpha=1.0, theta_l="bf16")
            mats.append(MatrixState(to_dev(inp.theta_g), K, to_dev(inp.q_in), 8, 64, dlcx.MMA_BF16))
            tls.append([to_dev(inp.theta_local(inp.theta_g, 1, i)) for i in range(K)])
        st = Stage(mats, synth.LR, synth.MU, fused=True, warm_start=True, streams=2,
                   measure_rank=True)
        load = torch.cuda.Stream(device=DEV)
        a = torch.randn(2048, 2048, device=DEV, dtype=torch.bfloat16)
        b = torch.randn(2048, 2048, device=DEV, dtype=torch.bfloat16)
        c = torch.empty(2048, 2048, device=DEV, dtype=torch.bfloat16)
        torch.cuda.synchronize()
        for _ in range(3):
            if busy:
                with torch.cuda.stream(load):
                    for _ in range(40):
                        torch.matmul(a, b, out=c)
            st.step(tls)
        torch.cuda.synchronize()
        return st

    alone, beside = run(False), run(True)
    for A, B in zip(alone.mats, beside.mats):
        assert torch.equal(A.theta_g, B.theta_g) and torch.equal(A.v, B.v)
        assert torch.equal(A.q_bar, B.q_bar) and torch.equal(A.p_hat, B.p_hat)
        for x, y in zip(A.ef, B.ef):
            assert torch.equal(x, y)
    assert torch.equal(alone.rprime_dev, beside.rprime_dev)
