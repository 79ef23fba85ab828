"""GPU parity, kernel by kernel: every step of the hot path is fed the SAME inputs as the CPU
oracle and compared element by element through the C ABI.

Bars: integer codes and scales of the quantiser bit-exact; floats rel-L2 <= 1e-5 on the fp32
paths (DLCX_MMA_FMA, DLCX_MMA_F32) and <= 2e-3 on the bf16 MFMA path.
"""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2506_21263_amd as dlcx
import synth
from oracle import ref
from gpu_util import DEV, GUARD, close, payload_buffers, rel_l2, to_dev, to_np, ws_for

pytestmark = pytest.mark.gpu

TOL = GUARD
MODES = [dlcx.MMA_FMA, dlcx.MMA_F32, dlcx.MMA_BF16]
MODE_IDS = ["mma_fma", "mma_f32", "mma_bf16"]


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ streaming kernels
@pytest.mark.parametrize("numel", [0, 1, 3, 4, 1023, 4096, 4099, 1 << 20, (1 << 20) + 7])
@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_delta_ef(numel, kind):
    g = rng(numel + 11)
    pad = numel + 8
    tg = (0.02 * g.standard_normal(pad)).astype(np.float32)
    e = (1e-3 * g.standard_normal(pad)).astype(np.float32)
    tl32 = (tg - 1e-3 * g.standard_normal(pad)).astype(np.float32)
    tl = synth.f32_to_bf16_bits(tl32) if kind == "bf16" else tl32
    want = ref.delta_ef(tg[:numel], tl[:numel], e[:numel]) if numel else np.zeros(0, np.float32)
    d_e = to_dev(e)
    dlcx.dlcx_delta_ef(to_dev(tg), to_dev(tl), d_e, numel=numel)
    got = to_np(d_e)
    assert np.array_equal(got[numel:], e[numel:]), "wrote past numel"
    if numel:  # (theta - theta_l) + e summed in fp64 and rounded once on both sides
        assert np.array_equal(got[:numel].view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("numel", [0, 4, 5, 4096, (1 << 20) + 3])
def test_outer_nesterov(numel):
    g = rng(numel + 5)
    pad = numel + 8
    th = (0.02 * g.standard_normal(pad)).astype(np.float32)
    v = (1e-3 * g.standard_normal(pad)).astype(np.float32)
    gr = (1e-3 * g.standard_normal(pad)).astype(np.float32)
    th_w, v_w = th[:numel].copy(), v[:numel].copy()
    if numel:
        ref.outer_nesterov(th_w, v_w, gr[:numel].copy(), synth.LR, synth.MU)
    d_th, d_v = to_dev(th), to_dev(v)
    dlcx.dlcx_outer_nesterov(d_th, d_v, to_dev(gr), synth.LR, synth.MU, numel=numel)
    got_th, got_v = to_np(d_th), to_np(d_v)
    assert np.array_equal(got_th[numel:], th[numel:]) and np.array_equal(got_v[numel:], v[numel:])
    if numel:
        assert rel_l2(got_th[:numel], th_w) <= 1e-6 and rel_l2(got_v[:numel], v_w) <= 1e-6


def test_outer_nesterov_three_steps_closed_form(golden):
    g = golden("nesterov_closed_form.txt")
    th = torch.zeros(8, device=DEV)
    v = torch.zeros(8, device=DEV)
    gr = torch.ones(8, device=DEV)
    for want in g["theta_t1_t2_t3"]:
        dlcx.dlcx_outer_nesterov(th, v, gr, g["lr"][0], g["mu"][0])
        assert np.allclose(to_np(th), want, rtol=3e-7)


# ------------------------------------------------------------------ quantiser
@pytest.mark.parametrize("qbits", [4, 8])
@pytest.mark.parametrize("group", [16, 32, 64, 128, 256])
def test_quantize_codes_and_scales_bit_exact(qbits, group):
    g = rng(qbits * 1000 + group)
    count = group * 1031  # ragged against the 1024-element workgroup
    x = (g.standard_normal(count) * np.exp(2 * g.standard_normal(count))).astype(np.float32)
    x[3 * group:4 * group] = 0.0                       # all-zero group
    x[5 * group:6 * group] = 1e-40                      # denormal group (below the cut)
    qmax = 2 ** (qbits - 1) - 1
    x[7 * group] = float(qmax)                          # exact ties: x * inv on .5 boundaries
    x[7 * group + 1:8 * group] = 0.0
    x[7 * group + 1:7 * group + 7] = [0.5, 1.5, 2.5, -0.5, -1.5, -2.5]
    codes_w, scales_w = ref.quantize(x, qbits, group)
    codes = torch.zeros(codes_w.size, device=DEV, dtype=torch.uint8)
    scales = torch.zeros(scales_w.size, device=DEV, dtype=torch.float32)
    dlcx.dlcx_quantize(to_dev(x), qbits, group, codes, scales)
    assert np.array_equal(to_np(scales).view(np.uint32), scales_w.view(np.uint32))
    assert np.array_equal(to_np(codes), codes_w)


@pytest.mark.parametrize("qbits,group,K", [(4, 64, 2), (4, 128, 4), (8, 64, 8), (4, 16, 1), (8, 256, 16),
                                           (4, 32, 3), (8, 128, 7)])
def test_dequant_average(qbits, group, K):
    g = rng(K * 7 + qbits)
    count = group * 517
    payloads = [ref.quantize((g.standard_normal(count) * (1 + k)).astype(np.float32), qbits, group)
                for k in range(K)]
    want = ref.dequant_average([p[0] for p in payloads], [p[1] for p in payloads], count, qbits, group)
    out = torch.zeros(count, device=DEV)
    dlcx.dlcx_dequant_average([to_dev(p[0]) for p in payloads], [to_dev(p[1]) for p in payloads],
                              count, qbits, group, out)
    # fp64 sum of exact products in worker order, one rounding: the same bits on both sides
    assert np.array_equal(to_np(out).view(np.uint32), want.view(np.uint32))


# ------------------------------------------------------------------ rank-r products
SHAPES = [  # (m, n, r, K, group): several tiles and ragged tails in both dimensions
    (512, 512, 8, 2, 64),
    (528, 336, 5, 3, 16),
    (208, 1040, 33, 1, 16),
    (1024, 768, 64, 4, 128),
    (640, 2048, 96, 2, 128),
    (2048, 512, 256, 1, 64),
    (4096, 320, 200, 8, 64),     # enough workgroups for the 128-row form of the P kernel
    # the two-role kernels with ragged rows and columns, a partial last stage and a partial last
    # basis block, at 2, 4 and 8 basis blocks
    (4240, 208, 40, 8, 16),
    (4112, 336, 72, 8, 16),
    (4112, 336, 130, 8, 16),
    # the smallest sizes the descriptor admits (one group per side, rank 1), the largest number
    # of workers, a rank equal to the smaller side
    (16, 16, 1, 1, 16),
    (32, 48, 16, 16, 16),
    (64, 48, 40, 2, 16),
]


def _lowrank_inputs(m, n, r, K, seed):
    inp = synth.MatrixInputs(m, n, K, r, seed=seed, sigma=1e-3, alpha=1.0)
    deltas = [inp.raw_pseudo_gradient(1, k).astype(np.float32) for k in range(K)]
    return inp, deltas


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("m,n,r,K,group", SHAPES)
def test_project_p_and_q(mma, m, n, r, K, group):
    inp, deltas = _lowrank_inputs(m, n, r, K, seed=m + n + r)
    d = dlcx.desc(m, n, r, 4, group, mma)
    ws = ws_for(d, K)
    d_deltas = [to_dev(x) for x in deltas]
    # P phase with the round-1 Gaussian basis
    want_p = [ref.project_p(x, inp.q_in) for x in deltas]
    outs = [torch.zeros(r, m, device=DEV) for _ in range(K)]
    dlcx.dlcx_project(d, dlcx.PHASE_P, d_deltas, to_dev(inp.q_in), outs, ws)
    for k in range(K):
        assert close(to_np(outs[k]), want_p[k], TOL[mma]), ("P", k)
    # Q phase with the oracle's orthonormal basis
    p_hat = ref.orthonormalize(np.mean(want_p, axis=0).astype(np.float32))
    want_q = [ref.project_q(x, p_hat) for x in deltas]
    outs = [torch.zeros(r, n, device=DEV) for _ in range(K)]
    dlcx.dlcx_project(d, dlcx.PHASE_Q, d_deltas, to_dev(p_hat), outs, ws)
    for k in range(K):
        assert close(to_np(outs[k]), want_q[k], TOL[mma]), ("Q", k)


# ranks above 64 in the fp16 form: (Q only: few rows) / (P and Q: the two-role P kernel is used)
SHAPES_F16 = [(640, 2048, 96, 2, 128), (2048, 512, 256, 1, 64), (4096, 320, 200, 8, 64),
              (4112, 336, 72, 8, 16), (4112, 336, 130, 8, 16)]


@pytest.mark.parametrize("m,n,r,K,group", SHAPES_F16)
def test_project_p_and_q_fp16_form(m, n, r, K, group):
    test_project_p_and_q(dlcx.MMA_F16, m, n, r, K, group)


def test_fp16_form_is_the_bf16_form_up_to_rank_64():
    m, n, r, K, group = 1024, 768, 64, 4, 128
    inp, deltas = _lowrank_inputs(m, n, r, K, seed=5)
    basis_q = rng(9).standard_normal((r, m)).astype(np.float32)
    outs = {}
    for mma in (dlcx.MMA_BF16, dlcx.MMA_F16):
        d = dlcx.desc(m, n, r, 4, group, mma)
        po = [torch.zeros(r, m, device=DEV) for _ in range(K)]
        qo = [torch.zeros(r, n, device=DEV) for _ in range(K)]
        dd = [to_dev(x) for x in deltas]
        dlcx.dlcx_project(d, dlcx.PHASE_P, dd, to_dev(inp.q_in), po, ws_for(d, K))
        dlcx.dlcx_project(d, dlcx.PHASE_Q, dd, to_dev(basis_q), qo, ws_for(d, K))
        outs[mma] = [to_np(x) for x in po + qo]
    for a, b in zip(outs[dlcx.MMA_BF16], outs[dlcx.MMA_F16]):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("case", ["in-range", "huge-element", "tiny", "zero"])
def test_fp16_form_stands_by_outside_its_range(case):
    """The fp16 launch records the largest |delta|; outside [2^-14, 15.99) the stand-by launch
    redoes the projection in the bf16 arithmetic, so the result is then that of DLCX_MMA_BF16 bit
    for bit -- a single element of 1e3 among values of 1e-3, a matrix of values around 1e-9, an
    all-zero matrix.  In range, the result is the fp16 one (close to, not equal to, the bf16 one)."""
    m, n, r, K, group = 4096, 320, 200, 8, 64
    inp, deltas = _lowrank_inputs(m, n, r, K, seed=77)
    if case == "huge-element":
        deltas[3][1234, 77] = 1.0e3
    elif case == "tiny":
        deltas = [(x * 1e-7).astype(np.float32) for x in deltas]
    elif case == "zero":
        deltas = [np.zeros_like(x) for x in deltas]
    d_deltas = [to_dev(x) for x in deltas]
    p_hat = ref.orthonormalize(ref.project_p(deltas[0] if case != "zero" else inp.theta_g, inp.q_in))
    res = {}
    for mma in (dlcx.MMA_BF16, dlcx.MMA_F16):
        d = dlcx.desc(m, n, r, 4, group, mma)
        ws = ws_for(d, K)
        po = [torch.zeros(r, m, device=DEV) for _ in range(K)]
        qo = [torch.zeros(r, n, device=DEV) for _ in range(K)]
        dlcx.dlcx_project(d, dlcx.PHASE_P, d_deltas, to_dev(inp.q_in), po, ws)
        dlcx.dlcx_project(d, dlcx.PHASE_Q, d_deltas, to_dev(p_hat), qo, ws)
        res[mma] = [to_np(x) for x in po + qo]
    same = all(np.array_equal(a.view(np.uint32), b.view(np.uint32))
               for a, b in zip(res[dlcx.MMA_BF16], res[dlcx.MMA_F16]))
    if case == "in-range":
        assert not same
        for a, b in zip(res[dlcx.MMA_BF16], res[dlcx.MMA_F16]):
            assert close(b, a, TOL[dlcx.MMA_F16])
        want = ref.project_q(deltas[2], p_hat)
        assert close(res[dlcx.MMA_F16][K + 2], want, TOL[dlcx.MMA_F16])
    else:
        assert same
        if case != "zero":
            want = ref.project_q(deltas[3], p_hat)
            assert rel_l2(res[dlcx.MMA_F16][K + 3], want) <= TOL[dlcx.MMA_BF16]


@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("m,n,r,K,group", SHAPES)
def test_decompress_and_error_buffer(mma, m, n, r, K, group):
    g = rng(m * 3 + n)
    p_hat = ref.orthonormalize(g.standard_normal((r, m)).astype(np.float32))
    q_bar = (g.standard_normal((r, n)) * np.arange(1, r + 1)[:, None] ** -1.0).astype(np.float32)
    deltas = [g.standard_normal((m, n)).astype(np.float32) * 0.1 for _ in range(K)]
    want = ref.reconstruct(p_hat, q_bar)
    want_e = [ref.ef_update(x.copy().reshape(-1), want.reshape(-1)).reshape(m, n) for x in deltas]
    d = dlcx.desc(m, n, r, 4, group, mma)
    out = torch.zeros(m, n, device=DEV)
    efs = [to_dev(x) for x in deltas]
    ws = ws_for(d, max(K, 1))
    dlcx.dlcx_decompress(d, to_dev(p_hat), to_dev(q_bar), out, efs, workspace=ws)
    assert close(to_np(out), want, TOL[mma])
    for k in range(K):
        # e = delta - delta_hat: compare the correction, not the (larger) buffer
        assert close(deltas[k] - to_np(efs[k]), deltas[k] - want_e[k], TOL[mma])
    # error buffers only (no materialised delta_hat) gives the same buffers
    efs2 = [to_dev(x) for x in deltas]
    dlcx.dlcx_decompress(d, to_dev(p_hat), to_dev(q_bar), None, efs2, workspace=ws)
    for k in range(K):
        assert torch.equal(efs2[k], efs[k])
    # fused with the outer update: same error buffers, and (theta, v) as the separate kernels give
    g2 = rng(7)
    th = (0.02 * g2.standard_normal((m, n))).astype(np.float32)
    v = (1e-3 * g2.standard_normal((m, n))).astype(np.float32)
    th_w, v_w = th.copy(), v.copy()
    ref.outer_nesterov(th_w.reshape(-1), v_w.reshape(-1), want.reshape(-1), synth.LR, synth.MU)
    efs3 = [to_dev(x) for x in deltas]
    d_th, d_v = to_dev(th), to_dev(v)
    dlcx.dlcx_decompress_apply(d, to_dev(p_hat), to_dev(q_bar), efs3, d_th, d_v, synth.LR, synth.MU,
                               workspace=ws)
    for k in range(K):
        assert torch.equal(efs3[k], efs[k])
    assert close(th - to_np(d_th), th - th_w, TOL[mma])
    assert close(to_np(d_v), v_w, TOL[mma])


# ------------------------------------------------------------------ compress = project + quantise
@pytest.mark.parametrize("mma", MODES, ids=MODE_IDS)
@pytest.mark.parametrize("qbits", [4, 8])
def test_compress_codes_are_the_quantiser_of_its_own_factor(mma, qbits):
    m, n, r, K, group = 1024, 768, 32, 3, 128
    inp, deltas = _lowrank_inputs(m, n, r, K, seed=99)
    d = dlcx.desc(m, n, r, qbits, group, mma)
    ws = ws_for(d, K)
    for phase, basis, L in ((dlcx.PHASE_P, inp.q_in, m),
                            (dlcx.PHASE_Q, ref.orthonormalize(rng(1).standard_normal((r, m)).astype(np.float32)), n)):
        codes, scales = payload_buffers(d, phase, K)
        dlcx.dlcx_compress_batched(d, phase, [to_dev(x) for x in deltas], to_dev(basis), codes, scales, ws)
        torch.cuda.synchronize()
        factors = to_np(ws[: K * r * L * 4].view(torch.float32)).reshape(K, r, L)
        for k in range(K):
            want_f = (ref.project_p if phase == dlcx.PHASE_P else ref.project_q)(deltas[k], basis)
            assert close(factors[k], want_f, TOL[mma])
            cw, sw = ref.quantize(factors[k], qbits, group)   # oracle quantiser on the GPU's factor
            assert np.array_equal(to_np(codes[k]), cw)
            assert np.array_equal(to_np(scales[k]).view(np.uint32), sw.view(np.uint32))
        # the single-worker entry point writes the same payload
        c1, s1 = payload_buffers(d, phase, 1)
        dlcx.dlcx_compress(d, phase, to_dev(deltas[1]), to_dev(basis), c1[0], s1[0], ws)
        assert torch.equal(c1[0], codes[1]) and torch.equal(s1[0], scales[1])


# ------------------------------------------------------------------ orthonormalisation
@pytest.mark.parametrize("L,r", [(64, 1), (512, 8), (528, 5), (2048, 64), (1040, 33), (4096, 128),
                                  (1024, 200), (2048, 256)])
def test_orthonormalize_matches_oracle(L, r):
    g = rng(L + r)
    # columns with very different norms and a decaying spectrum (warm-started basis)
    U = synth.orthonormal_columns(g, L, r)
    W = synth.orthonormal_columns(g, r, r)
    s = np.arange(1, r + 1, dtype=np.float64) ** -1.5
    A = ((U * s) @ W.T * (np.arange(1, r + 1) ** -2.0)).T.astype(np.float32)
    A = np.ascontiguousarray(A)
    want = ref.orthonormalize(A)
    d_A = to_dev(A)
    ws = torch.empty(dlcx.dlcx_workspace_bytes(dlcx.desc(L, L, r, 4, 16), 1), device=DEV, dtype=torch.uint8)
    dlcx.dlcx_orthonormalize(L, r, d_A, ws)
    got = to_np(d_A).astype(np.float64)
    assert np.abs(got @ got.T - np.eye(r)).max() <= 1e-5
    cond = np.linalg.cond(A.astype(np.float64))
    assert rel_l2(got, want) <= max(1e-5, 4e-7 * cond), cond


def test_orthonormalize_degenerate_columns():
    L, r = 256, 6
    g = rng(3)
    A = g.standard_normal((r, L)).astype(np.float32)
    A[1] = 0.0
    A[4] = -3.0 * A[2]
    want = ref.orthonormalize(A)
    d_A = to_dev(A)
    ws = torch.empty(dlcx.dlcx_workspace_bytes(dlcx.desc(L, L, r, 4, 16), 1), device=DEV, dtype=torch.uint8)
    dlcx.dlcx_orthonormalize(L, r, d_A, ws)
    got = to_np(d_A)
    assert np.all(got[1] == 0) and np.all(got[4] == 0)
    assert rel_l2(got, want) <= 1e-5
    z = torch.zeros(3, L, device=DEV)
    dlcx.dlcx_orthonormalize(L, 3, z, ws)
    assert not to_np(z).any()


# ------------------------------------------------------------------ effective rank
@pytest.mark.parametrize("alpha,want", [(0.5, 241), (1.0, 49), (2.0, 3)])
def test_effective_rank_prescribed_spectra(alpha, want):
    n, r = 512, 256
    V = synth.orthonormal_columns(rng(1), n, r)
    W = synth.orthonormal_columns(rng(2), r, r)          # rotate: Gram is dense
    sig = np.arange(1, r + 1, dtype=np.float64) ** (-alpha)
    q_bar = np.ascontiguousarray(((V * sig) @ W.T).T.astype(np.float32))
    assert ref.effective_rank(q_bar, 0.99) == want
    out = torch.zeros(1, device=DEV, dtype=torch.int32)
    ws = torch.empty(dlcx.dlcx_workspace_bytes(dlcx.desc(n, n, r, 4, 16), 1), device=DEV, dtype=torch.uint8)
    dlcx.dlcx_effective_rank(n, r, to_dev(q_bar), 0.99, out, ws)
    assert int(out.item()) == want


@pytest.mark.parametrize("n,r", [(64, 1), (128, 7), (528, 33), (1024, 64), (768, 128), (512, 129),
                                 (512, 130), (1024, 192), (512, 255), (768, 256)])
def test_effective_rank_random_and_zero(n, r):
    g = rng(n + r)
    q = (g.standard_normal((r, n)) * (np.arange(1, r + 1)[:, None] ** -1.2)).astype(np.float32)
    ws = torch.empty(dlcx.dlcx_workspace_bytes(dlcx.desc(n, n, r, 4, 16), 1), device=DEV, dtype=torch.uint8)
    out = torch.full((1,), -1, device=DEV, dtype=torch.int32)
    for tau in (0.5, 0.9, 0.99, 1.0):
        dlcx.dlcx_effective_rank(n, r, to_dev(q), tau, out, ws)
        assert int(out.item()) == ref.effective_rank(q, tau), tau
    dlcx.dlcx_effective_rank(n, r, torch.zeros(r, n, device=DEV), 0.99, out, ws)
    assert int(out.item()) == 0
    if r >= 8:  # rank-deficient Gram: repeated, zero and low-rank columns
        q2 = q.copy()
        q2[5] = q2[3]
        q2[6] = 0.0
        q2[r // 2:] = (g.standard_normal((r - r // 2, 3)) @ g.standard_normal((3, n))).astype(np.float32)
        for tau in (0.9, 0.999, 1.0):
            dlcx.dlcx_effective_rank(n, r, to_dev(q2), tau, out, ws)
            want = ref.effective_rank(q2, tau)
            # at tau = 1 the count depends on eigenvalues at rounding level: not compared
            if tau < 1.0:
                assert int(out.item()) == want, tau


def test_select_rank_stage_value_and_window():
    # three matrices with known r' (3, 49, zero matrix -> rmin 4): mean 56/3 = 18.67 -> 19
    n, r = 512, 64
    mats = []
    for alpha in (2.0, 1.0):
        V = synth.orthonormal_columns(rng(5), n, 256)
        sig = np.arange(1, 257, dtype=np.float64) ** (-alpha)
        mats.append(np.ascontiguousarray((V * sig).T.astype(np.float32)))
    descs = [dlcx.desc(n, n, 256, 4, 16), dlcx.desc(n, n, 256, 4, 16), dlcx.desc(n, n, r, 4, 16)]
    q_bars = [to_dev(mats[0]), to_dev(mats[1]), torch.zeros(r, n, device=DEV)]
    assert [ref.effective_rank(x, 0.99) for x in mats] == [3, 49]
    ws = torch.empty(dlcx.dlcx_select_rank_workspace_bytes(descs), device=DEV, dtype=torch.uint8)
    hist = (C.c_int32 * 5)(256, 256, 256, 256, 0)
    rp, r_next, H = dlcx.dlcx_select_rank(descs, q_bars, 0.99, hist, 5, 5, 256, 4, 256, 125, workspace=ws)
    assert rp == 19
    want_r, want_H = ref.adagradcmp([256, 256, 256, 256, 19], 5, 5, 256, 4, 256, 125)
    assert (r_next, H) == (want_r, want_H)


def test_batched_orthonormalize_and_rank_mixed_shapes():
    # 70 factors of different lengths and ranks in one call (more than one launch chunk of 64):
    # same results as the one-matrix entry points, which are checked against the oracle above.
    g = rng(4242)
    shapes = [(256 + 16 * (i % 9), 8 + (i * 7) % 57) for i in range(70)]      # (L, r)
    shapes[3] = (2048, 200)                                                   # global-memory path
    descs, ps, qs, ps_single = [], [], [], []
    for L, r in shapes:
        descs.append(dlcx.desc(L, L, r, 4, 16))
        a = (g.standard_normal((r, L)) * (np.arange(1, r + 1)[:, None] ** -1.0)).astype(np.float32)
        ps.append(to_dev(a))
        ps_single.append(to_dev(a))
        qs.append(to_dev(a))
    ws = torch.empty(dlcx.dlcx_batched_workspace_bytes(descs), device=DEV, dtype=torch.uint8)
    out = torch.zeros(len(descs), device=DEV, dtype=torch.int32)
    dlcx.dlcx_effective_rank_batched(descs, qs, 0.9, out, ws)
    dlcx.dlcx_orthonormalize_batched(descs, ps, ws)
    one = torch.zeros(1, device=DEV, dtype=torch.int32)
    for i, (L, r) in enumerate(shapes):
        w1 = torch.empty(dlcx.dlcx_workspace_bytes(descs[i], 1), device=DEV, dtype=torch.uint8)
        dlcx.dlcx_orthonormalize(L, r, ps_single[i], w1)
        assert torch.equal(ps[i], ps_single[i]), i
        dlcx.dlcx_effective_rank(L, r, qs[i], 0.9, one, w1)
        assert int(one.item()) == int(out[i].item()), i
    for i in (0, 3, 17, 69):
        assert int(out[i].item()) == ref.effective_rank(to_np(qs[i]), 0.9)
        assert rel_l2(to_np(ps[i]), ref.orthonormalize(to_np(qs[i]))) <= 1e-5
