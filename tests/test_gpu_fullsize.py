"""Parity at the benchmark's full matrix sizes, in the launch configuration bench.py times
(bf16 MFMA mode, fused round kernel, K = 4, r = 64, int4 / 128, bf16 local replicas).

A full matrix of the ~100B-class stage is too large for the oracle to sweep step by step in a
test, so the oracle computes (with its unchanged single-threaded routines, called from a thread
pool on disjoint outputs) the full factors of one round, and every GPU entry point is then fed
the ORACLE's inputs and checked on sampled outputs: whole quantisation groups of the factors
(codes bit for bit, boundary flips by one step allowed), and sampled rows of delta, theta and v.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import paper_2506_21263_amd as dlcx
import synth
from oracle import ref
from gpu_util import (DEV, GUARD, close, code_mismatch_report, payload_buffers, rel_l2, to_dev,
                      to_np, ws_for)

pytestmark = pytest.mark.gpu

POOL = 16
K, R, QBITS, GROUP, MMA = 4, 64, 4, 128, dlcx.MMA_BF16
TOL = GUARD[dlcx.MMA_BF16]


def _bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def _oracle_full_p(deltas, q_in):
    """P_k = delta_k Q_in for all rows: row chunks in parallel, each output from one oracle call."""
    m = deltas[0].shape[0]
    step = max(128, m // (2 * POOL) // 128 * 128)
    jobs = [(k, i0) for k in range(len(deltas)) for i0 in range(0, m, step)]
    out = [np.empty((q_in.shape[0], m), np.float32) for _ in deltas]

    def run(job):
        k, i0 = job
        out[k][:, i0:i0 + step] = ref.project_p(np.ascontiguousarray(deltas[k][i0:i0 + step]), q_in)

    with ThreadPoolExecutor(POOL) as ex:
        list(ex.map(run, jobs))
    return out


def _oracle_q_columns(deltas, p_hat, cols):
    """Q_k[:, j] for the given columns j (one oracle call per column and worker)."""
    out = [np.empty((p_hat.shape[0], len(cols)), np.float32) for _ in deltas]
    jobs = [(k, a) for k in range(len(deltas)) for a in range(len(cols))]

    def run(job):
        k, a = job
        out[k][:, a] = ref.project_q_row(deltas[k], p_hat, int(cols[a]))

    with ThreadPoolExecutor(POOL) as ex:
        list(ex.map(run, jobs))
    return out


def _check_groups(codes_gpu, scales_gpu, factor_ref, L, groups, what, r=R, ref_offset=0):
    """Bit-compare the payload of whole groups (along L) of every factor column; factor_ref
    holds the reference factor from element ref_offset of each column on."""
    G = GROUP
    flips = 0
    for g in groups:
        blk = np.ascontiguousarray(factor_ref[:, g * G - ref_offset:(g + 1) * G - ref_offset])
        cw, sw = ref.quantize(blk.reshape(-1), QBITS, G)
        got_c = np.stack([codes_gpu[(c * L + g * G) // 2:(c * L + (g + 1) * G) // 2]
                          for c in range(r)]).reshape(-1)
        got_s = np.array([scales_gpu[(c * L) // G + g] for c in range(r)], np.float32)
        assert close(got_s, sw, TOL), what
        nb, ok = code_mismatch_report(got_c, cw, blk, sw, r * G, QBITS, G, ref.unpack_codes)
        assert ok, (what, g, "code mismatch that is not a one-step boundary flip")
        flips += nb
    return flips


@pytest.mark.timeout(400)
@pytest.mark.parametrize("m,n", [(8192, 1024), (8192, 8192), (8192, 28672), (28672, 8192)])
def test_full_size_matrix_sampled(m, n):
    print("full-size case %dx%d" % (m, n), flush=True)
    rs = np.random.default_rng(m + n)
    sigma = float(synth.noise_sigma(2, m, n))
    t = synth.torch_matrix_inputs(m, n, K, R, seed=synth.seed_for(77, m, n), sigma=sigma, alpha=1.2,
                                  theta_l="bf16", device=DEV)
    theta0 = t["theta_g"].cpu().numpy()
    tl_bits = [_bits(x) for x in t["theta_l"]]
    q_in = t["q_in"].cpu().numpy()
    d = dlcx.desc(m, n, R, QBITS, GROUP, MMA)
    ws = ws_for(d, K)

    # ---------------- round 1 on the oracle: delta, P, P_hat, sampled Q, (full Q_bar later)
    zeros = np.zeros(m * n, np.float32)
    deltas = [ref.delta_ef(theta0.reshape(-1), b.reshape(-1), zeros).reshape(m, n) for b in tl_bits]
    P = _oracle_full_p(deltas, q_in)
    payload_p = [ref.quantize(p, QBITS, GROUP) for p in P]
    p_bar = ref.dequant_average([c for c, _ in payload_p], [s for _, s in payload_p], R * m, QBITS,
                                GROUP).reshape(R, m)
    p_hat = ref.orthonormalize(p_bar)

    # ---------------- GPU round 1, the fused entry point the bench uses (r_prev = 0)
    efs = [torch.zeros(m, n, device=DEV) for _ in range(K)]
    th, v = t["theta_g"].clone(), torch.zeros(m, n, device=DEV)
    codes, scales = payload_buffers(d, dlcx.PHASE_P, K)
    dlcx.dlcx_ef_delta_apply_compress(d, 0, None, None, t["theta_l"], efs, th, v, synth.LR, synth.MU,
                                      t["q_in"], codes, scales, ws)
    torch.cuda.synchronize()
    assert torch.equal(th, t["theta_g"]) and not bool(v.any())       # nothing applied at t = 1
    rows = np.sort(rs.choice(m, 24, replace=False))
    for k in range(K):
        got = efs[k][torch.from_numpy(rows).to(DEV)].cpu().numpy()
        assert rel_l2(got, deltas[k][rows]) <= 1e-6, ("delta", k)
    groups_m = rs.choice(m // GROUP, 6, replace=False)
    flips = 0
    for k in range(K):
        flips += _check_groups(to_np(codes[k]), to_np(scales[k]), P[k], m, groups_m, ("P", k))
    # average + orthonormalisation from the oracle's payloads
    d_p_hat = torch.zeros(R, m, device=DEV)
    dlcx.dlcx_average(d, dlcx.PHASE_P, [to_dev(c) for c, _ in payload_p],
                      [to_dev(s) for _, s in payload_p], d_p_hat, ws)
    cond = np.linalg.cond(p_bar.astype(np.float64))
    assert rel_l2(to_np(d_p_hat), p_hat) <= max(1e-5, 4e-7 * cond), cond
    # Q phase from the oracle's basis: whole groups of columns
    codes_q, scales_q = payload_buffers(d, dlcx.PHASE_Q, K)
    efs_oracle = [to_dev(x) for x in deltas]
    dlcx.dlcx_compress_batched(d, dlcx.PHASE_Q, efs_oracle, to_dev(p_hat), codes_q, scales_q, ws)
    torch.cuda.synchronize()
    groups_n = rs.choice(n // GROUP, 3, replace=False)
    cols = np.concatenate([np.arange(g * GROUP, (g + 1) * GROUP) for g in groups_n])
    Qs = _oracle_q_columns(deltas, p_hat, cols)
    for k in range(K):
        cg, sg = to_np(codes_q[k]), to_np(scales_q[k])
        for a, g in enumerate(groups_n):
            blk = np.ascontiguousarray(Qs[k][:, a * GROUP:(a + 1) * GROUP])
            cw, sw = ref.quantize(blk.reshape(-1), QBITS, GROUP)
            got_c = np.stack([cg[(c * n + g * GROUP) // 2:(c * n + (g + 1) * GROUP) // 2]
                              for c in range(R)]).reshape(-1)
            got_s = np.array([sg[(c * n) // GROUP + g] for c in range(R)], np.float32)
            assert close(got_s, sw, TOL), ("Q scales", k)
            nb, ok = code_mismatch_report(got_c, cw, blk, sw, R * GROUP, QBITS, GROUP,
                                          ref.unpack_codes)
            assert ok, ("Q", k, g)
            flips += nb
    assert flips <= 2e-3 * K * R * GROUP * (len(groups_m) + len(groups_n)), flips
    del efs_oracle

    # ---------------- round 2, fused: error buffers, new delta, outer update, sampled
    # The previous average for the check is any rank-r pair: the oracle's P_hat and a Q_bar made
    # of the sampled columns' structure is not available in full, so use a seeded Q_bar instead.
    q_bar = (rs.standard_normal((R, n)) * (np.arange(1, R + 1)[:, None] ** -1.0) * 1e-2).astype(np.float32)
    tl2 = [synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(b) + np.float32(1e-4) * rs.standard_normal((m, n)).astype(np.float32))
           for b in tl_bits[:K]]
    efs2 = [to_dev(x) for x in deltas]
    th2, v2 = t["theta_g"].clone(), torch.zeros(m, n, device=DEV)
    v_host = (1e-4 * rs.standard_normal((m, n))).astype(np.float32)
    v2.copy_(to_dev(v_host))
    codes2, scales2 = payload_buffers(d, dlcx.PHASE_P, K)
    dlcx.dlcx_ef_delta_apply_compress(d, R, to_dev(p_hat), to_dev(q_bar), [to_dev(x) for x in tl2],
                                      efs2, th2, v2, synth.LR, synth.MU, to_dev(q_bar), codes2,
                                      scales2, ws)
    torch.cuda.synchronize()
    idx = torch.from_numpy(rows).to(DEV)
    d_hat_rows = ref.reconstruct(np.ascontiguousarray(p_hat[:, rows]), q_bar)          # (24, n)
    th_w, v_w = theta0[rows].copy(), v_host[rows].copy()
    new_delta = []
    for k in range(K):
        e = deltas[k][rows].copy()
        ref.ef_update(e.reshape(-1), d_hat_rows.reshape(-1))
        new_delta.append(ref.delta_ef(theta0[rows].reshape(-1), np.ascontiguousarray(tl2[k][rows]).reshape(-1),
                                      e.reshape(-1)).reshape(len(rows), n))
    ref.outer_nesterov(th_w.reshape(-1), v_w.reshape(-1), d_hat_rows.reshape(-1), synth.LR, synth.MU)
    for k in range(K):
        got = efs2[k][idx].cpu().numpy()
        assert close(got, new_delta[k], TOL), ("delta round 2", k)
        # the part the kernel subtracts is the decompressed average: check it at the MFMA bar
        base = deltas[k][rows] + (theta0[rows] - synth.bf16_bits_to_f32(tl2[k][rows]))
        assert close(base - got, d_hat_rows, TOL), ("delta_hat via delta", k)
    assert close(theta0[rows] - th2[idx].cpu().numpy(), theta0[rows] - th_w, TOL)
    assert close(v2[idx].cpu().numpy(), v_w, TOL)
    # P phase of round 2 on the sampled groups needs the full new delta: rows of whole groups
    g0 = int(groups_m[0])
    grp_rows = np.arange(g0 * GROUP, (g0 + 1) * GROUP)
    d_hat_g = ref.reconstruct(np.ascontiguousarray(p_hat[:, grp_rows]), q_bar)
    for k in range(K):
        e = deltas[k][grp_rows].copy()
        ref.ef_update(e.reshape(-1), d_hat_g.reshape(-1))
        nd = ref.delta_ef(theta0[grp_rows].reshape(-1), np.ascontiguousarray(tl2[k][grp_rows]).reshape(-1),
                          e.reshape(-1)).reshape(GROUP, n)
        p_rows = ref.project_p(nd, q_bar)                                             # (r, 128)
        cw, sw = ref.quantize(np.ascontiguousarray(p_rows).reshape(-1), QBITS, GROUP)
        cg, sg = to_np(codes2[k]), to_np(scales2[k])
        got_s = np.array([sg[(c * m) // GROUP + g0] for c in range(R)], np.float32)
        got_c = np.stack([cg[(c * m + g0 * GROUP) // 2:(c * m + (g0 + 1) * GROUP) // 2]
                          for c in range(R)]).reshape(-1)
        assert close(got_s, sw, TOL), ("P round 2 scales", k)
        nb, ok = code_mismatch_report(got_c, cw, p_rows, sw, R * GROUP, QBITS, GROUP, ref.unpack_codes)
        assert ok and nb <= 0.02 * R * GROUP, ("P round 2 payload", k, nb)


def test_quantise_only_step_full_size_sampled_groups():
    # The quantise-only sweep on a tensor the size of the largest matrix of the stage (28672 x
    # 8192 = 234.9 M elements, K = 4, int4 / 128, bf16 replicas), three outer steps running free.
    # Every operation of that step is local to a group of 128 elements, so the oracle run on a
    # sample of whole groups (first, last and 3000 drawn at random) must reproduce the GPU's
    # values there bit for bit.  The replicas are synthetic and do not depend on GPU results.
    from oracle import pipeline
    numel, Kq, group, T = 28672 * 8192, 4, 128, 3
    gen = torch.Generator(device=DEV)
    gen.manual_seed(4242)
    theta = 0.02 * torch.randn(numel, device=DEV, generator=gen)
    v = torch.zeros_like(theta)
    ef = [torch.zeros(numel, device=DEV) for _ in range(Kq)]
    codes = [torch.zeros(numel // 2, device=DEV, dtype=torch.uint8) for _ in range(Kq)]
    scales = [torch.zeros(numel // group, device=DEV) for _ in range(Kq)]
    ngroups = numel // group
    rng = np.random.default_rng(7)
    gsel = np.unique(np.concatenate([[0, 1, ngroups - 2, ngroups - 1],
                                     rng.integers(0, ngroups, 3000)])).astype(np.int64)
    eidx = (torch.from_numpy(gsel).to(DEV)[:, None] * group +
            torch.arange(group, device=DEV)[None, :]).reshape(-1)
    gidx = torch.from_numpy(gsel).to(DEV)
    theta0_s = theta[eidx].cpu().numpy()
    orc = pipeline.TensorOracle(theta0_s, Kq, 4, group, synth.LR, synth.MU)
    theta0_dev = theta.clone()
    for t in range(1, T + 1):
        tl = []
        for i in range(Kq):
            g = 1e-3 * torch.randn(numel, device=DEV, generator=gen) * (1.0 + 4.0 * (i == t % Kq))
            tl.append((theta0_dev - g).to(torch.bfloat16))
        orc.step([_bits(x[eidx]) for x in tl])
        dlcx.dlcx_quant_round(numel, 4, group, tl, ef, theta, v, synth.LR, synth.MU,
                              None if t == 1 else codes, None if t == 1 else scales, codes, scales)
        torch.cuda.synchronize()
        cidx = (gidx[:, None] * (group // 2) +
                torch.arange(group // 2, device=DEV)[None, :]).reshape(-1)
        for i in range(Kq):
            assert np.array_equal(codes[i][cidx].cpu().numpy(), orc.codes[i]), (t, i)
            assert np.array_equal(scales[i][gidx].cpu().numpy().view(np.uint32),
                                  orc.scales[i].view(np.uint32)), (t, i)
            assert np.array_equal(ef[i][eidx].cpu().numpy().view(np.uint32),
                                  orc.ef[i].view(np.uint32)), (t, i)
        assert np.array_equal(theta[eidx].cpu().numpy().view(np.uint32), orc.theta.view(np.uint32)), t
        assert np.array_equal(v[eidx].cpu().numpy().view(np.uint32), orc.v.view(np.uint32)), t
    assert orc.n_applied == T - 1 and not np.array_equal(orc.theta, theta0_s)


def test_flat_tensors_beyond_2_31_elements():
    # Largest sizes: a flat tensor of 2^31 + 4736 elements (+ 3 for the entry points that take a
    # ragged tail), where every 32-bit element index overflows.  All these steps are local to an
    # element or to a group of 128, so the oracle run on three windows (the start, across 2^31,
    # the end with the tail) must reproduce the GPU there: bit for bit for delta, codes, scales
    # and the quantise-only step, to 1e-6 for the fp32 Nesterov kernel.
    from oracle import pipeline
    group = 128
    numel = 2 ** 31 + group * 37
    total = numel + 3
    win = [(0, 8192), (2 ** 31 - 8192, 2 ** 31 + 4096), (numel - 8192, total)]
    gen = torch.Generator(device=DEV)
    gen.manual_seed(31)

    def sample(x, upto=total):
        return [x[a:min(b, upto)].cpu().numpy() for a, b in win]

    theta = torch.empty(total, device=DEV).normal_(0.0, 0.02, generator=gen)
    e = torch.empty(total, device=DEV).normal_(0.0, 1e-3, generator=gen)
    tl = torch.empty(total, device=DEV).normal_(0.0, 1e-3, generator=gen).neg_().add_(theta)
    tl = tl.to(torch.bfloat16)
    th_s, e_s, tl_s = sample(theta), sample(e), [_bits(x[a:b]) for x in [tl] for a, b in win]
    # ---- pseudo-gradient with error compensation
    dlcx.dlcx_delta_ef(theta, tl, e)
    torch.cuda.synchronize()
    d_s = sample(e)
    for w in range(3):
        want = ref.delta_ef(th_s[w], tl_s[w], e_s[w])
        assert np.array_equal(d_s[w].view(np.uint32), want.view(np.uint32)), ("delta_ef", w)
    # ---- quantiser on the first numel elements (whole groups)
    codes = torch.zeros(numel // 2, device=DEV, dtype=torch.uint8)
    scales = torch.zeros(numel // group, device=DEV)
    dlcx.dlcx_quantize(e, 4, group, codes, scales, count=numel)
    torch.cuda.synchronize()
    for w, (a, b) in enumerate(win):
        b = min(b, numel)
        cw, sw = ref.quantize(d_s[w][: b - a], 4, group)
        assert np.array_equal(codes[a // 2:b // 2].cpu().numpy(), cw), ("codes", w)
        assert np.array_equal(scales[a // group:b // group].cpu().numpy().view(np.uint32),
                              sw.view(np.uint32)), ("scales", w)
    del codes, scales
    # ---- outer Nesterov step with delta as the gradient
    v = torch.empty(total, device=DEV).normal_(0.0, 1e-3, generator=gen)
    v_s = sample(v)
    dlcx.dlcx_outer_nesterov(theta, v, e, synth.LR, synth.MU)
    torch.cuda.synchronize()
    th2, v2 = sample(theta), sample(v)
    for w in range(3):
        tw, vw = th_s[w].copy(), v_s[w].copy()
        ref.outer_nesterov(tw, vw, d_s[w], synth.LR, synth.MU)
        assert rel_l2(th2[w], tw) <= 1e-6 and rel_l2(v2[w], vw) <= 1e-6, ("nesterov", w)
        assert not np.array_equal(th2[w], th_s[w])
    del tl, e
    # ---- the quantise-only outer step, K = 2, two steps running free on numel elements
    Kq = 2
    theta = theta[:numel]
    v = v[:numel].zero_()
    theta0 = theta.clone()
    ef = [torch.zeros(numel, device=DEV) for _ in range(Kq)]
    codes = [torch.zeros(numel // 2, device=DEV, dtype=torch.uint8) for _ in range(Kq)]
    scales = [torch.zeros(numel // group, device=DEV) for _ in range(Kq)]
    qwin = [(a, min(b, numel)) for a, b in win]
    cat = lambda x: np.concatenate([x[a:b].cpu().numpy() for a, b in qwin])
    orc = pipeline.TensorOracle(cat(theta), Kq, 4, group, synth.LR, synth.MU)
    for t in (1, 2):
        tls = []
        for i in range(Kq):
            g = torch.empty(numel, device=DEV).normal_(0.0, 1e-3 * (1 + i + t), generator=gen)
            tls.append(g.neg_().add_(theta0).to(torch.bfloat16))
            del g
        orc.step([np.concatenate([_bits(x[a:b]) for a, b in qwin]) for x in tls])
        dlcx.dlcx_quant_round(numel, 4, group, tls, ef, theta, v, synth.LR, synth.MU,
                              None if t == 1 else codes, None if t == 1 else scales, codes, scales)
        torch.cuda.synchronize()
        for i in range(Kq):
            got_c = np.concatenate([codes[i][a // 2:b // 2].cpu().numpy() for a, b in qwin])
            got_s = np.concatenate([scales[i][a // group:b // group].cpu().numpy() for a, b in qwin])
            assert np.array_equal(got_c, orc.codes[i]), (t, i)
            assert np.array_equal(got_s.view(np.uint32), orc.scales[i].view(np.uint32)), (t, i)
            assert np.array_equal(cat(ef[i]).view(np.uint32), orc.ef[i].view(np.uint32)), (t, i)
        assert np.array_equal(cat(theta).view(np.uint32), orc.theta.view(np.uint32)), t
        assert np.array_equal(cat(v).view(np.uint32), orc.v.view(np.uint32)), t
        del tls
    assert orc.n_applied == 1


@pytest.mark.timeout(400)
def test_matrix_beyond_2_31_elements():
    # Largest sizes on the low-rank path: one 65536 x 32896 matrix (2.156 G elements, element
    # 2^31 sits in row 65280), K = 1, r = 8, bf16 replica, the fused entry point of the bench.
    # Round 1 and the Q phase against the oracle on whole groups at the start, across the 2^31
    # boundary and at the end; round 2 (feedback, new delta, outer update) on sampled rows there.
    m, n, r, Kb = 65536, 32896, 8, 1
    assert m * n > 2 ** 31
    print("matrix %dx%d" % (m, n), flush=True)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(65536)
    # theta ~ N(0, 0.02^2); pseudo-gradient = rank-12 part with a 1/k spectrum + small noise
    theta = torch.empty(m, n, device=DEV).normal_(0.0, 0.02, generator=gen)
    U = torch.linalg.qr(torch.randn(m, 12, device=DEV, generator=gen))[0]
    V = torch.linalg.qr(torch.randn(n, 12, device=DEV, generator=gen))[0]
    sv = 1.0 / torch.arange(1, 13, device=DEV)
    g = (U * sv) @ V.T
    g.add_(torch.empty(m, n, device=DEV).normal_(0.0, 2e-5, generator=gen))
    tl = (theta - g).to(torch.bfloat16)
    del g, U, V
    q_in_t = torch.randn(r, n, device=DEV, generator=gen)
    theta0 = theta.cpu().numpy()
    tl_bits = _bits(tl)
    q_in = q_in_t.cpu().numpy()
    d = dlcx.desc(m, n, r, QBITS, GROUP, MMA)
    ws = ws_for(d, Kb)
    rows = np.array([0, 1, 31, 32, 65279, 65280, 65281, 65407, 65408, m - 33, m - 2, m - 1])

    # ---- oracle, round 1
    delta = ref.delta_ef(theta0.reshape(-1), tl_bits.reshape(-1),
                         np.zeros(m * n, np.float32)).reshape(m, n)
    P = _oracle_full_p([delta], q_in)
    cp, sp = ref.quantize(P[0], QBITS, GROUP)
    p_bar = ref.dequant_average([cp], [sp], r * m, QBITS, GROUP).reshape(r, m)
    p_hat = ref.orthonormalize(p_bar)

    # ---- GPU round 1, fused entry point (r_prev = 0)
    efs = [torch.zeros(m, n, device=DEV)]
    th, v = theta.clone(), torch.zeros(m, n, device=DEV)
    codes, scales = payload_buffers(d, dlcx.PHASE_P, Kb)
    dlcx.dlcx_ef_delta_apply_compress(d, 0, None, None, [tl], efs, th, v, synth.LR, synth.MU,
                                      q_in_t, codes, scales, ws)
    torch.cuda.synchronize()
    assert torch.equal(th, theta) and not bool(v.any())
    idx = torch.from_numpy(rows).to(DEV)
    assert rel_l2(efs[0][idx].cpu().numpy(), delta[rows]) <= 1e-6
    groups_m = [0, 65280 // GROUP, m // GROUP - 1]          # rows 65280.. hold element 2^31
    flips = _check_groups(to_np(codes[0]), to_np(scales[0]), P[0], m, groups_m, "P", r=r)
    d_p_hat = torch.zeros(r, m, device=DEV)
    dlcx.dlcx_average(d, dlcx.PHASE_P, [to_dev(cp)], [to_dev(sp)], d_p_hat, ws)
    cond = np.linalg.cond(p_bar.astype(np.float64))
    assert rel_l2(to_np(d_p_hat), p_hat) <= max(1e-5, 4e-7 * cond), cond
    # ---- Q phase from the oracle's basis: first and last group of columns
    codes_q, scales_q = payload_buffers(d, dlcx.PHASE_Q, Kb)
    dlcx.dlcx_compress_batched(d, dlcx.PHASE_Q, efs, to_dev(p_hat), codes_q, scales_q, ws)
    torch.cuda.synchronize()
    for gq in (0, n // GROUP - 1):
        cols = np.arange(gq * GROUP, (gq + 1) * GROUP)
        Qs = _oracle_q_columns([delta], p_hat, cols)
        flips += _check_groups(to_np(codes_q[0]), to_np(scales_q[0]), Qs[0], n, [gq], "Q", r=r,
                               ref_offset=gq * GROUP)
    assert flips <= 2e-3 * r * GROUP * 5 + 2, flips

    # ---- round 2, fused, with a seeded previous Q_bar: sampled rows
    rs = np.random.default_rng(5)
    q_bar = (rs.standard_normal((r, n)) * (np.arange(1, r + 1)[:, None] ** -1.0) * 1e-2).astype(np.float32)
    tl2 = (tl.float() + torch.empty(m, n, device=DEV).normal_(0.0, 1e-4, generator=gen)).to(torch.bfloat16)
    v.normal_(0.0, 1e-4, generator=gen)
    v_rows = v[idx].cpu().numpy()
    tl2_rows = _bits(tl2[idx])
    codes2, scales2 = payload_buffers(d, dlcx.PHASE_P, Kb)
    dlcx.dlcx_ef_delta_apply_compress(d, r, to_dev(p_hat), to_dev(q_bar), [tl2], efs, th, v,
                                      synth.LR, synth.MU, to_dev(q_bar), codes2, scales2, ws)
    torch.cuda.synchronize()
    d_hat_rows = ref.reconstruct(np.ascontiguousarray(p_hat[:, rows]), q_bar)
    e = delta[rows].copy()
    ref.ef_update(e.reshape(-1), d_hat_rows.reshape(-1))
    nd = ref.delta_ef(theta0[rows].reshape(-1), np.ascontiguousarray(tl2_rows).reshape(-1),
                      e.reshape(-1)).reshape(len(rows), n)
    th_w, v_w = theta0[rows].copy(), v_rows.copy()
    ref.outer_nesterov(th_w.reshape(-1), v_w.reshape(-1), d_hat_rows.reshape(-1), synth.LR, synth.MU)
    got = efs[0][idx].cpu().numpy()
    assert close(got, nd, TOL)
    base = delta[rows] + (theta0[rows] - synth.bf16_bits_to_f32(tl2_rows))
    assert close(base - got, d_hat_rows, TOL)
    assert close(theta0[rows] - th[idx].cpu().numpy(), theta0[rows] - th_w, TOL)
    assert close(v[idx].cpu().numpy(), v_w, TOL)
    # the P payload of round 2 for the last group of rows (all beyond element 2^31)
    g0 = m // GROUP - 1
    grp = np.arange(g0 * GROUP, m)
    gidx = torch.from_numpy(grp).to(DEV)
    d_hat_g = ref.reconstruct(np.ascontiguousarray(p_hat[:, grp]), q_bar)
    e = delta[grp].copy()
    ref.ef_update(e.reshape(-1), d_hat_g.reshape(-1))
    nd_g = ref.delta_ef(theta0[grp].reshape(-1), np.ascontiguousarray(_bits(tl2[gidx])).reshape(-1),
                        e.reshape(-1)).reshape(GROUP, n)
    p_rows = ref.project_p(nd_g, q_bar)
    flips2 = _check_groups(to_np(codes2[0]), to_np(scales2[0]), p_rows, m, [g0], "P round 2", r=r,
                           ref_offset=g0 * GROUP)
    assert flips2 <= 0.02 * r * GROUP
