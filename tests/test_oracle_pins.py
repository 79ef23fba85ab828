"""Pins of the CPU oracle against things other than itself.

Each test names the passage of the paper (or the piece of mathematics) that fixes
the expected value.  A plausible mistake anywhere in the oracle (dropped term,
wrong sign or index, transposed operand) is meant to fail at least one of these.
"""
import numpy as np
import pytest

import synth
from oracle import pipeline, ref
from conftest import read_golden

RNG = np.random.default_rng(20250621)


def rel(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


# --------------------------------------------------------------------------- delta / EF
def test_delta_ef_hand_values_and_sign():
    # Alg. 2: delta = (theta_global - theta_local) + e.  Hand values; a swapped sign fails.
    tg = np.array([1.0, -2.0, 0.5, 0.0], np.float32)
    tl = np.array([0.25, -3.0, 0.5, 1.0], np.float32)
    e = np.array([0.5, 0.125, -1.0, 0.0], np.float32)
    assert ref.delta_ef(tg, tl, e).tolist() == [1.25, 1.125, -1.0, -1.0]


def test_delta_ef_bf16_widening_is_exact():
    # bf16 bit patterns: 0x3F80 = 1.0, 0xC000 = -2.0, 0x3E00 = 0.125, 0x0000 = 0
    tl = np.array([0x3F80, 0xC000, 0x3E00, 0x0000], np.uint16)
    tg = np.zeros(4, np.float32)
    e = np.zeros(4, np.float32)
    assert ref.delta_ef(tg, tl, e).tolist() == [-1.0, 2.0, -0.125, 0.0]
    x = RNG.standard_normal(1000).astype(np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(ref.delta_ef(tg[:1].repeat(1000), bits, np.zeros(1000, np.float32)), -back)


# --------------------------------------------------------------------------- LOWRANK
def _lowrank_once(M_list, q_in):
    """One shared-basis iteration without quantisation; returns (P_hat, Q_bar, M_hat)."""
    P = [ref.project_p(M, q_in) for M in M_list]
    p_hat = ref.orthonormalize(pipeline._mean64(P))
    Q = [ref.project_q(M, p_hat) for M in M_list]
    q_bar = pipeline._mean64(Q)
    return p_hat, q_bar, ref.reconstruct(p_hat, q_bar)


def test_projections_against_unit_vectors():
    # P = M Q_in with Q_in = unit vector e_j picks column j of M; Q = M^T P_hat with
    # P_hat = e_i picks row i.  Catches a transposed operand on a non-square matrix.
    m, n = 5, 9
    M = RNG.standard_normal((m, n)).astype(np.float32)
    q_in = np.zeros((2, n), np.float32)
    q_in[0, 3] = 1.0
    q_in[1, 7] = 2.0
    P = ref.project_p(M, q_in)
    assert np.array_equal(P[0], M[:, 3]) and np.array_equal(P[1], 2 * M[:, 7])
    p_hat = np.zeros((2, m), np.float32)
    p_hat[0, 4] = 1.0
    p_hat[1, 1] = -1.0
    Q = ref.project_q(M, p_hat)
    assert np.array_equal(Q[0], M[4]) and np.array_equal(Q[1], -M[1])
    assert np.array_equal(ref.project_q_row(M, p_hat, 6), Q[:, 6])
    # reconstruction of an outer product
    R = ref.reconstruct(p_hat, Q)
    expect = np.zeros((m, n), np.float32)
    expect[4] = M[4]
    expect[1] = M[1]
    assert np.array_equal(R, expect)


def test_exact_reconstruction_when_rank_fits():
    # rank(M) <= r  =>  one iteration with a generic basis reproduces M.
    m, n, r = 48, 80, 6
    A = RNG.standard_normal((m, r))
    B = RNG.standard_normal((r, n))
    M = (A @ B).astype(np.float32)
    q_in = RNG.standard_normal((r, n)).astype(np.float32)
    _, _, M_hat = _lowrank_once([M], q_in)
    # factors are stored in fp32: the error is eps_fp32 times the condition number of P
    assert rel(M_hat, M) < 1e-4
    # full rank r = min(m, n)
    m, n = 12, 20
    M = RNG.standard_normal((m, n)).astype(np.float32)
    q_in = RNG.standard_normal((m, n)).astype(np.float32)
    _, _, M_hat = _lowrank_once([M], q_in)
    assert rel(M_hat, M) < 1e-4


def test_truncated_svd_special_case_config0_numbers():
    # M = U diag(1/k) V^T (512 x 512), basis = V[:, :8]  =>  M_hat is the best rank-8
    # approximation and ||M - M_hat||_F^2 = sum_{k>8} k^-2 = 0.1155608 of 1.6429828.
    inp = synth.MatrixInputs(512, 512, 1, 8, seed=7, sigma=0.0, alpha=1.0)
    s = inp.spectrum()
    M64 = (inp.U * s) @ inp.V.T
    M = M64.astype(np.float32)
    q_in = np.ascontiguousarray(inp.V[:, :8].T.astype(np.float32))
    p_hat, q_bar, M_hat = _lowrank_once([M], q_in)
    err2 = np.sum((M.astype(np.float64) - M_hat) ** 2)
    tot2 = np.sum(M.astype(np.float64) ** 2)
    assert abs(err2 - 0.1155608) < 2e-6
    assert abs(tot2 - 1.6429828) < 2e-6
    best = (inp.U[:, :8] * s[:8]) @ inp.V[:, :8].T
    assert rel(M_hat, best) < 1e-5
    # library cross-check: numpy's SVD gives the same best approximation
    u, sv, vt = np.linalg.svd(M64)
    assert rel(M_hat, (u[:, :8] * sv[:8]) @ vt[:8]) < 1e-5


def test_projector_identities_and_orthonormality():
    m, n, r, K = 96, 64, 5, 3
    Ms = [RNG.standard_normal((m, n)).astype(np.float32) for _ in range(K)]
    q_in = RNG.standard_normal((r, n)).astype(np.float32)
    p_hat, q_bar, M_hat = _lowrank_once(Ms, q_in)
    Mbar = np.mean([M.astype(np.float64) for M in Ms], axis=0)
    G = p_hat.astype(np.float64) @ p_hat.T.astype(np.float64)
    assert np.abs(G - np.eye(r)).max() < 1e-6
    resid = Mbar - M_hat
    assert abs(np.sum(resid * M_hat)) < 1e-5 * np.sum(Mbar ** 2)
    assert abs(np.sum(Mbar ** 2) - np.sum(M_hat.astype(np.float64) ** 2) - np.sum(resid ** 2)) \
        < 1e-5 * np.sum(Mbar ** 2)
    # M_hat = P_hat P_hat^T Mbar
    assert rel(M_hat, p_hat.T.astype(np.float64) @ (p_hat.astype(np.float64) @ Mbar)) < 1e-5


def test_allreduce_linearity_and_identical_workers():
    # "can be implemented using the AllReduce": with a shared basis the factors are linear
    # in delta, so project-then-average equals average-then-project.
    m, n, r, K = 40, 56, 4, 4
    Ms = [RNG.standard_normal((m, n)).astype(np.float32) for _ in range(K)]
    q_in = RNG.standard_normal((r, n)).astype(np.float32)
    Mbar = np.mean([M.astype(np.float64) for M in Ms], axis=0).astype(np.float32)
    _, _, a = _lowrank_once(Ms, q_in)
    _, _, b = _lowrank_once([Mbar], q_in)
    assert rel(a, b) < 5e-6
    _, _, c = _lowrank_once([Ms[0]] * K, q_in)
    _, _, d = _lowrank_once([Ms[0]], q_in)
    assert rel(c, d) < 1e-6


def test_subspace_iteration_converges_to_truncated_svd():
    # repeated rounds on a fixed matrix with warm start Q_in <- Q_bar
    inp = synth.MatrixInputs(64, 48, 1, 4, seed=11, sigma=0.0, alpha=2.0)
    s = inp.spectrum()
    M = ((inp.U * s) @ inp.V.T).astype(np.float32)
    q_in = inp.q_in
    for _ in range(12):
        _, q_bar, M_hat = _lowrank_once([M], q_in)
        q_in = q_bar
    best = (inp.U[:, :4] * s[:4]) @ inp.V[:, :4].T
    assert rel(M_hat, best) < 1e-4


def test_power_iterations_within_a_round_are_subspace_iteration():
    # iters power iterations inside one round act on the round's own pseudo-gradients: with the
    # quantiser off they are subspace iteration on the mean matrix, so the residual falls
    # monotonically towards the Eckart-Young bound sqrt(sum_{k>r} sigma_k^2) (numpy's SVD of the
    # mean), and the decompressed average approaches the best rank-r approximation.
    m, n, r, K = 72, 56, 4, 3
    inp = synth.MatrixInputs(m, n, K, r, seed=23, sigma=2e-3, alpha=1.5)
    theta = inp.theta_g
    tl = [inp.theta_local(theta, 1, i) for i in range(K)]
    Mbar = np.mean([theta.astype(np.float64) - x for x in tl], axis=0)
    u, sv, vt = np.linalg.svd(Mbar)
    floor = np.sqrt(np.sum(sv[r:] ** 2))
    best = (u[:, :r] * sv[:r]) @ vt[:r]
    errs = []
    for iters in (1, 2, 3, 6, 40):
        orc = pipeline.MatrixOracle(theta, K, inp.q_in, None, 1, iters=iters)
        orc.step(tl)
        assert np.array_equal(orc.theta, theta)           # nothing is applied at t = 1
        errs.append(np.linalg.norm(Mbar - orc.delta_hat()))
        assert errs[-1] >= floor * (1 - 1e-6)
    assert all(a > b for a, b in zip(errs, errs[1:]))     # every further iteration helps
    assert errs[-1] <= floor * (1 + 1e-4)
    assert rel(orc.delta_hat(), best) < 2e-3
    # the second iteration starts from the first one's Q average (a hand-over to anything else,
    # the round's input basis say, would repeat the first iteration instead)
    orc = pipeline.MatrixOracle(theta, K, inp.q_in, None, 1, iters=2)
    orc.step(tl)
    Ms = [d for d in orc.trace["delta"]]
    _, q1, _ = _lowrank_once(Ms, inp.q_in)
    p2, q2, _ = _lowrank_once(Ms, q1)
    assert np.array_equal(orc.trace["q_bar"], q1) and np.array_equal(orc.trace["q_in@1"], q1)
    assert np.array_equal(orc.p_hat, p2) and np.array_equal(orc.q_bar, q2)


# --------------------------------------------------------------------------- orthonormalize
def test_orthonormalize_matches_householder_qr():
    m, r = 30, 7
    A = RNG.standard_normal((r, m)).astype(np.float32)
    got = ref.orthonormalize(A)
    q, rr = np.linalg.qr(A.T.astype(np.float64))  # LAPACK Householder
    q = q * np.sign(np.diag(rr))
    assert np.abs(got - q.T).max() < 1e-6
    R = got.astype(np.float64) @ A.T.astype(np.float64)  # P_hat^T P = R
    assert np.all(np.diag(R) > 0)
    assert np.abs(np.tril(R, -1)).max() < 1e-5
    assert rel(got.T.astype(np.float64) @ R, A.T) < 1e-6


def test_orthonormalize_degenerate_columns():
    m = 16
    A = RNG.standard_normal((4, m)).astype(np.float32)
    A[1] = 0.0           # zero column
    A[3] = 2.0 * A[0]    # duplicate direction
    got = ref.orthonormalize(A)
    assert np.all(got[1] == 0) and np.all(got[3] == 0)
    assert abs(np.linalg.norm(got[0]) - 1) < 1e-6 and abs(np.linalg.norm(got[2]) - 1) < 1e-6
    assert abs(float(got[0].astype(np.float64) @ got[2])) < 1e-6
    assert np.all(ref.orthonormalize(np.zeros((3, m), np.float32)) == 0)


def test_orthonormalize_ill_conditioned():
    # cond ~ 1e5: columns still orthonormal to fp32 level and span preserved
    m, r = 200, 6
    U = synth.orthonormal_columns(RNG, m, r)
    W = synth.orthonormal_columns(RNG, r, r)
    A = ((U * np.logspace(0, -5, r)) @ W.T).T.astype(np.float32)
    got = ref.orthonormalize(np.ascontiguousarray(A)).astype(np.float64)
    assert np.abs(got @ got.T - np.eye(r)).max() < 1e-6
    q, rr = np.linalg.qr(A.T.astype(np.float64))
    q = q * np.sign(np.diag(rr))
    assert np.abs(got - q.T).max() < 1e-5


# --------------------------------------------------------------------------- quantiser
@pytest.mark.parametrize("qbits,group", [(4, 64), (4, 128), (8, 64), (4, 16)])
def test_quantize_half_step_bound_and_range(qbits, group):
    count = group * 37
    x = (RNG.standard_normal(count) * np.exp(RNG.standard_normal(count))).astype(np.float32)
    codes, scales = ref.quantize(x, qbits, group)
    qmax = 2 ** (qbits - 1) - 1
    ci = ref.unpack_codes(codes, count, qbits)
    assert ci.min() >= -qmax and ci.max() <= qmax
    xh = ref.dequantize(codes, scales, count, qbits, group)
    s_el = np.repeat(scales, group).astype(np.float64)
    assert np.all(np.abs(x.astype(np.float64) - xh) <= 0.5 * s_el * (1 + 2.0 ** -20))
    # the element of largest magnitude maps to +-qmax, and scale = amax / qmax
    xg = x.reshape(-1, group)
    am = np.abs(xg).max(axis=1)
    assert np.array_equal(scales, (am / np.float32(qmax)).astype(np.float32))
    idx = np.abs(xg).argmax(axis=1)
    top = ci.reshape(-1, group)[np.arange(xg.shape[0]), idx]
    assert np.array_equal(np.abs(top), np.full_like(top, qmax))
    assert np.array_equal(np.sign(top), np.sign(xg[np.arange(xg.shape[0]), idx]).astype(top.dtype))
    # re-quantising the dequantised values reproduces the codes
    codes2, scales2 = ref.quantize(xh, qbits, group)
    assert np.array_equal(codes2, codes) and np.array_equal(scales2, scales)


def test_quantize_every_int4_code_and_nibble_order():
    # group of 16: x = k * 0.5 for k = -7..7 plus one zero => amax 3.5, scale 0.5, codes = k
    ks = list(range(-7, 8)) + [0]
    x = np.array([0.5 * k for k in ks], np.float32)
    codes, scales = ref.quantize(x, 4, 16)
    assert scales.tolist() == [0.5]
    assert ref.unpack_codes(codes, 16, 4).tolist() == ks
    # element 2j in the low nibble, 2j+1 in the high nibble, two's complement
    expect = [((ks[2 * j + 1] & 0xF) << 4) | (ks[2 * j] & 0xF) for j in range(8)]
    assert codes.tolist() == expect
    assert expect[0] == 0xA9  # (-7 -> 0x9 low, -6 -> 0xA high)


def test_quantize_round_half_even_zero_group_and_int8():
    # amax = 7 => inv = 1: values on .5 boundaries round to even
    x = np.array([7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5] + [0.0] * 8, np.float32)
    codes, scales = ref.quantize(x, 4, 16)
    assert scales.tolist() == [1.0]
    assert ref.unpack_codes(codes, 16, 4)[:8].tolist() == [7, 0, 2, 2, 0, -2, -2, 4]
    z = np.zeros(32, np.float32)
    codes, scales = ref.quantize(z, 4, 16)
    assert not codes.any() and not scales.any()
    tiny = np.full(16, 1e-40, np.float32)  # below the 2^-100 cut: treated as a zero group
    codes, scales = ref.quantize(tiny, 8, 16)
    assert not codes.any() and not scales.any()
    x8 = np.array([127.0, -127.0, 1.0, -1.0, 63.5, 64.5, 0.0, 0.0] * 2, np.float32)
    codes, scales = ref.quantize(x8, 8, 16)
    assert ref.unpack_codes(codes, 16, 8)[:6].tolist() == [127, -127, 1, -1, 64, 64]


def test_average_hand_example_and_identity():
    # two workers, int8, group 16: mean of dequantised payloads, in worker order
    a = np.zeros(16, np.float32)
    b = np.zeros(16, np.float32)
    a[0], a[1] = 127.0, 2.0
    b[0], b[1] = -254.0, 4.0       # scale 2
    ca, sa = ref.quantize(a, 8, 16)
    cb, sb = ref.quantize(b, 8, 16)
    out = ref.dequant_average([ca, cb], [sa, sb], 16, 8, 16)
    assert out[:2].tolist() == [(127.0 - 254.0) / 2, (2.0 + 4.0) / 2]
    x = RNG.standard_normal(128).astype(np.float32)
    c, s = ref.quantize(x, 4, 64)
    assert np.array_equal(ref.dequant_average([c], [s], 128, 4, 64), ref.dequantize(c, s, 128, 4, 64))


# --------------------------------------------------------------------------- Nesterov, delay
def test_nesterov_closed_form_2x2():
    g = read_golden("nesterov_closed_form.txt")
    lr, mu = g["lr"][0], g["mu"][0]
    theta = np.zeros((2, 2), np.float32)
    v = np.zeros((2, 2), np.float32)
    grad = np.ones((2, 2), np.float32)
    for t, want in enumerate(g["theta_t1_t2_t3"], start=1):
        ref.outer_nesterov(theta.reshape(-1), v.reshape(-1), grad.reshape(-1), lr, mu)
        assert np.allclose(theta, want, rtol=2e-7, atol=0)
        closed = -lr * (t / (1 - mu) - mu ** 2 * (1 - mu ** t) / (1 - mu) ** 2)
        assert np.allclose(theta, closed, rtol=2e-7, atol=0)
    # a different gradient per element scales linearly (2x2 with distinct entries)
    theta = np.array([[1.0, -1.0], [0.5, 2.0]], np.float32)
    t0 = theta.copy()
    v = np.zeros((2, 2), np.float32)
    grad = np.array([[1.0, -2.0], [0.0, 0.25]], np.float32)
    for _ in range(3):
        ref.outer_nesterov(theta.reshape(-1), v.reshape(-1), grad.reshape(-1), lr, mu)
    assert np.allclose(theta, t0 - 5.6343 * grad, rtol=1e-6)


def _run_rounds(inp, T, qbits, group, K, alpha_by_round=None):
    orc = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, qbits, group, synth.LR, synth.MU)
    sum_g = [np.zeros((inp.m, inp.n), np.float64) for _ in range(K)]
    sum_dhat = np.zeros((inp.m, inp.n), np.float64)
    thetas = [orc.theta.copy()]
    for t in range(1, T + 1):
        tl = [inp.theta_local(orc.theta, t, i) for i in range(K)]
        for i in range(K):
            sum_g[i] += orc.theta.astype(np.float64) - tl[i].astype(np.float64)
        orc.step(tl)
        orc.set_basis(orc.q_bar)
        sum_dhat += orc.delta_hat()
        thetas.append(orc.theta.copy())
    return orc, sum_g, sum_dhat, thetas


@pytest.mark.parametrize("qbits", [None, 4])
def test_error_feedback_telescoping(qbits):
    # e^{t+1}_i = delta^t_i - Delta^t and delta^t_i = g^t_i + e^t_i  =>
    # sum_t Delta^t + e^{T+1}_i = sum_t g^t_i + e^1_i for every worker, any compressor.
    inp = synth.MatrixInputs(64, 128, 3, 4, seed=3, sigma=1e-3, alpha=1.0)
    T, K = 4, 3
    orc, sum_g, sum_dhat, _ = _run_rounds(inp, T, qbits, 64, K)
    d_hat = orc.delta_hat()
    for i in range(K):
        e_next = orc.ef[i].astype(np.float64) - d_hat  # e^{T+1}_i, not yet formed by step()
        assert rel(sum_dhat + e_next, sum_g[i]) < 1e-6 * T


def test_one_step_delay_schedule():
    # nothing applied at t = 1 (theta^1 == theta^0 bitwise); after T rounds T-1 updates.
    inp = synth.MatrixInputs(64, 64, 2, 4, seed=5, sigma=1e-3, alpha=1.0)
    orc, _, _, thetas = _run_rounds(inp, 3, 4, 64, 2)
    assert np.array_equal(thetas[1], thetas[0])
    assert not np.array_equal(thetas[2], thetas[1])
    assert orc.n_applied == 2


def test_delta_is_formed_before_theta_is_overwritten():
    # 1x... hand example of the ordering inside round 2: delta^2 = theta^1 - theta_l^2 + e^2
    # must use theta^1, not theta^2.  m = n = 16 so that one int8 group fits; only [0,0] is used.
    m = n = 16
    theta0 = np.zeros((m, n), np.float32)
    q_in = np.zeros((1, n), np.float32)
    q_in[0, 0] = 1.0
    orc = pipeline.MatrixOracle(theta0, 1, q_in, None, 16, lr=0.5, mu=0.0)
    tl1 = theta0.copy()
    tl1[0, 0] = -1.0                 # g^1 = theta^0 - theta_l = +1 at [0,0]
    orc.step([tl1])
    assert orc.delta_hat()[0, 0] == pytest.approx(1.0, abs=1e-6)
    tl2 = theta0.copy()              # replica unchanged in round 2: g^2 = theta^1 - 0 = 0
    orc.set_basis(q_in)
    orc.step([tl2])
    # e^2 = delta^1 - Delta^1 = 0 ; delta^2 = (theta^1 - tl2) + e^2 = 0 at [0,0]
    assert orc.trace["delta"][0][0, 0] == pytest.approx(0.0, abs=1e-6)
    # and theta^2 = theta^1 - lr * Delta^1 = -0.5
    assert orc.theta[0, 0] == pytest.approx(-0.5, abs=1e-6)


# --------------------------------------------------------------------------- rank selection
def test_adagradcmp_window_rule_hand_vectors():
    g = read_golden("adagradcmp_window.txt")
    c, r1, H1 = int(g["c"][0]), int(g["r1"][0]), int(g["H1"][0])
    hist = [int(x) for x in g["rprime"]]
    for t in range(1, 9):
        r, H = ref.adagradcmp(hist, t, c, r1, 4, r1, H1)
        assert r == int(g["r_t"][t - 1]) and H == int(g["H_t"][t - 1]), t
    # clamps
    assert ref.adagradcmp([1] * 5, 5, 5, 256, 4, 256, 125)[0] == 4
    assert ref.adagradcmp([300] * 5, 5, 5, 256, 4, 256, 125)[0] == 256


@pytest.mark.parametrize("alpha,want", [(0.5, 241), (1.0, 49), (2.0, 3)])
def test_effective_rank_prescribed_orthogonal_columns(alpha, want):
    # Q_bar with orthogonal columns of norm k^-alpha: Gram is diagonal, eigenvalues k^-2alpha,
    # r' = smallest k with sum_{i<=k} >= 0.99 sum  (241 / 49 / 3 over 256 columns).
    n, r = 512, 256
    V = synth.orthonormal_columns(np.random.default_rng(1), n, r)
    perm = np.random.default_rng(2).permutation(r)   # order of columns must not matter
    sig = np.arange(1, r + 1, dtype=np.float64) ** (-alpha)
    q_bar = np.ascontiguousarray((V * sig)[:, perm].T.astype(np.float32))
    assert ref.effective_rank(q_bar, 0.99) == want
    assert ref.effective_rank(np.zeros((8, 64), np.float32), 0.99) == 0
    assert pipeline.stage_rprime([0, 3, 4], 4) == 4      # (4 + 3 + 4) / 3 = 3.67 -> 4


def test_gram_eigenvalues_match_lapack():
    n, r = 96, 12
    q = RNG.standard_normal((r, n)).astype(np.float32)
    got = ref.gram_eigenvalues(q)
    want = np.linalg.eigvalsh(q.astype(np.float64) @ q.T.astype(np.float64))[::-1]
    assert np.allclose(got, want, rtol=1e-10, atol=1e-10 * want[0])
    # rotated known spectrum: Q_bar = V diag(sigma) W^T has Gram eigenvalues sigma^2
    V = synth.orthonormal_columns(RNG, n, r)
    W = synth.orthonormal_columns(RNG, r, r)
    sig = np.linspace(3.0, 0.1, r)
    q = np.ascontiguousarray(((V * sig) @ W.T).T.astype(np.float32))
    assert np.allclose(ref.gram_eigenvalues(q), sig ** 2, rtol=1e-5)


# --------------------------------------------------------------------------- accounting
def test_payload_accounting_against_paper_numbers():
    g = read_golden("compression_accounting.txt")
    m, n, r = int(g["m"][0]), int(g["n"][0]), int(g["r"][0])
    assert (m + n) * r / (m * n) == g["factor_fraction"][0]
    nb, ns = ref.payload_bytes((m + n) * r, 4, 128)
    fp16_bytes = 2 * (m + n) * r
    assert fp16_bytes / nb == g["int4_vs_fp16"][0]
    assert g["int4_vs_fp16"][0] * g["H1"][0] == g["ratio_opt"][0]
    assert 2 * g["int4_vs_fp16"][0] * g["H1"][0] == g["ratio_107b"][0]
    gb = 2 * (3 - 1) / 3 * 100e9 * 4 / 1e9
    assert abs(gb - g["allreduce_gb"][0]) < 0.05
    assert abs(gb / 0.125 / 3600 - g["allreduce_hours"][0]) < 0.01


def test_compression_error_is_a_contraction():
    # Assumption "Compression Error": ||C(x) - x||^2 <= omega^2 ||x||^2 with omega < 1.
    inp = synth.MatrixInputs(128, 128, 2, 8, seed=9, sigma=1e-3, alpha=1.0)
    orc = pipeline.MatrixOracle(inp.theta_g, 2, inp.q_in, 4, 64)
    tl = [inp.theta_local(orc.theta, 1, i) for i in range(2)]
    orc.step(tl)
    mean_delta = np.mean([d.astype(np.float64) for d in orc.trace["delta"]], axis=0)
    err = np.sum((orc.delta_hat() - mean_delta) ** 2)
    assert err < np.sum(mean_delta ** 2)


# --------------------------------------------------------------------------- quantise-only step
def _tensor_rounds(numel, K, T, qbits, group, seed, requant=False, kind="f32"):
    rng = np.random.default_rng(seed)
    theta0 = (0.02 * rng.standard_normal(numel)).astype(np.float32)
    orc = pipeline.TensorOracle(theta0, K, qbits, group, synth.LR, synth.MU, requant=requant)
    sum_g = [np.zeros(numel, np.float64) for _ in range(K)]
    sum_dhat = np.zeros(numel, np.float64)
    thetas = [orc.theta.copy()]
    for t in range(1, T + 1):
        tl = []
        for i in range(K):
            g = 1e-2 * rng.standard_normal(numel) * (1.0 + rng.uniform(0, 3, numel) ** 4)
            x = (orc.theta.astype(np.float64) - g).astype(np.float32)
            if kind == "bf16":
                x = synth.f32_to_bf16_bits(x)
                sum_g[i] += orc.theta.astype(np.float64) - synth.bf16_bits_to_f32(x)
            else:
                sum_g[i] += orc.theta.astype(np.float64) - x
            tl.append(x)
        orc.step(tl)
        sum_dhat += orc.delta_hat()
        thetas.append(orc.theta.copy())
    return orc, sum_g, sum_dhat, thetas


@pytest.mark.parametrize("requant", [False, True])
def test_tensor_step_telescoping_and_delay(requant):
    # The error-feedback identity holds for any compressor, so it pins the order of the
    # error-buffer update and the pseudo-gradient of Alg. 2 without reference to the quantiser.
    T, K = 4, 3
    orc, sum_g, sum_dhat, thetas = _tensor_rounds(1024, K, T, 4, 64, seed=11, requant=requant,
                                                  kind="bf16")
    d_hat = orc.delta_hat().astype(np.float64)
    for i in range(K):
        e_next = orc.ef[i].astype(np.float64) - d_hat
        assert rel(sum_dhat + e_next, sum_g[i]) < 1e-6 * T
    assert np.array_equal(thetas[1], thetas[0])      # nothing applied at t = 1
    assert not np.array_equal(thetas[2], thetas[1])
    assert orc.n_applied == T - 1


@pytest.mark.parametrize("qbits,group", [(4, 64), (8, 16)])
def test_tensor_step_single_worker_half_step_bound(qbits, group):
    # K = 1: Delta is the decoded payload, so the error buffer of the next round is the
    # quantisation residual, at most half a step of its group.
    orc, _, _, _ = _tensor_rounds(512, 1, 2, qbits, group, seed=12)
    delta = orc.ef[0]
    resid = np.abs(delta.astype(np.float64) - orc.delta_hat())
    qmax = 2 ** (qbits - 1) - 1
    amax = np.abs(delta).reshape(-1, group).max(axis=1)
    bound = np.repeat(amax / qmax / 2 * (1 + 2.0 ** -20), group)
    assert np.all(resid <= bound)
    assert resid.max() > 0


def test_tensor_step_exact_grid_follows_nesterov_closed_form():
    # Pseudo-gradients that sit exactly on the int8 grid (multiples of 2^-7, one element at
    # 127 * 2^-7 per group) pass the quantiser unchanged: e stays 0 and theta follows the closed
    # form of SGD with Nesterov momentum for a constant gradient, one round late.
    g = read_golden("nesterov_closed_form.txt")
    lr, mu = g["lr"][0], g["mu"][0]
    numel, group = 64, 16
    grad = (RNG.integers(-126, 127, numel) / 128.0).astype(np.float32)
    grad[::group] = 127.0 / 128.0
    theta0 = np.zeros(numel, np.float32)
    orc = pipeline.TensorOracle(theta0, 1, 8, group, lr, mu)
    for t in range(1, 5):
        tl = (orc.theta.astype(np.float64) - grad).astype(np.float32)
        orc.step([tl])
        # from round 3 on theta is off the grid, so the replica difference carries one fp32
        # rounding of theta; the codes are unchanged and the residual stays at that level
        assert np.allclose(orc.trace["delta"][0], grad, rtol=0, atol=1e-6)
        applied = t - 1
        closed = -lr * (applied / (1 - mu) - mu ** 2 * (1 - mu ** applied) / (1 - mu) ** 2)
        assert np.allclose(orc.theta, closed * grad, rtol=3e-6, atol=1e-6)
    # first round on an all-zero state is exact: Delta == grad bit for bit, residual zero
    orc = pipeline.TensorOracle(theta0, 1, 8, group, lr, mu)
    orc.step([(-grad).astype(np.float32)])
    assert np.array_equal(orc.delta_hat(), grad)


def test_tensor_step_mean_is_taken_over_workers_hand_example():
    # two workers, int8, one group of 16: worker 0 moves element 0 by -1, worker 1 by -3
    # (replica = theta - g) => delta = (1, 3), each exactly representable => Delta[0] = 2.
    theta0 = np.zeros(16, np.float32)
    tl0, tl1 = theta0.copy(), theta0.copy()
    tl0[0], tl1[0] = -1.0, -3.0
    orc = pipeline.TensorOracle(theta0, 2, 8, 16, lr=0.5, mu=0.0)
    orc.step([tl0, tl1])
    assert orc.delta_hat()[0] == 2.0
    assert np.all(orc.delta_hat()[1:] == 0.0)
    orc.step([theta0.copy(), theta0.copy()])       # replicas did not move in round 2
    assert orc.theta[0] == -1.0                      # theta^2 = theta^1 - 0.5 * 2
    # e_i = delta_i - Delta = (-1, +1); round 2 forms delta against theta^1 = 0
    assert orc.trace["delta"][0][0] == -1.0 and orc.trace["delta"][1][0] == 1.0


def test_requantized_mean_is_a_fixed_point_and_within_half_a_step():
    # Re-encoding a mean to q bits: the decoder output is a fixed point of the quantiser, the
    # error is at most half a step of the mean's own group, and with one worker (the mean is
    # already a decoded payload) nothing changes.
    x = RNG.standard_normal(4096).astype(np.float32)
    for qbits, group in ((4, 128), (8, 64)):
        y = pipeline.requantize(x, qbits, group)
        assert np.array_equal(pipeline.requantize(y, qbits, group), y)
        qmax = 2 ** (qbits - 1) - 1
        step = np.repeat(np.abs(x).reshape(-1, group).max(axis=1) / qmax, group)
        assert np.all(np.abs(x.astype(np.float64) - y) <= step / 2 * (1 + 2.0 ** -20))
    a, _, _, _ = _tensor_rounds(512, 1, 3, 4, 64, seed=13, requant=False)
    b, _, _, _ = _tensor_rounds(512, 1, 3, 4, 64, seed=13, requant=True)
    assert np.array_equal(a.theta, b.theta) and np.array_equal(a.ef[0], b.ef[0])


def test_requantized_factor_average_changes_only_within_the_bound():
    inp = synth.MatrixInputs(64, 128, 3, 4, seed=21, sigma=1e-3, alpha=1.0)
    tl = [inp.theta_local(inp.theta_g, 1, i) for i in range(3)]
    plain = pipeline.MatrixOracle(inp.theta_g, 3, inp.q_in, 4, 64)
    req = pipeline.MatrixOracle(inp.theta_g, 3, inp.q_in, 4, 64, requant=True)
    plain.step(tl)
    req.step(tl)
    # P phase: same payloads, the re-encoded mean differs from the mean by <= half a step
    pb, rb = plain.trace["p_bar"], req.trace["p_bar"]
    step = np.repeat(np.abs(pb).reshape(-1, 64).max(axis=1) / 7, 64).reshape(pb.shape)
    assert np.all(np.abs(pb.astype(np.float64) - rb) <= step / 2 * (1 + 2.0 ** -20))
    assert not np.array_equal(pb, rb)


# --------------------------------------------------------------------------- communication model
def test_comm_model_reproduces_the_papers_worked_example():
    # Sec. 2.4.1: 100B parameters in FP32, 3 clusters, 1 Gbps, H = 500 steps of 1 s.
    from oracle import planner
    g = read_golden("compression_accounting.txt")
    payload = 100e9 * 4
    between_gb = 2 * (3 - 1) * payload / 3 / 1e9
    assert abs(between_gb - g["allreduce_gb"][0]) < 0.05
    hours = planner.comm_seconds(payload, 3, 1e9) / 3600
    assert abs(hours - g["allreduce_hours"][0]) < 0.01
    local = g["local_steps"][0] * g["step_seconds"][0] / 3600
    assert abs(local - g["local_hours"][0]) < 0.01
    assert abs((hours - local) - g["idle_hours"][0]) < 0.01
    assert planner.comm_seconds(payload, 1, 1e9) == 0.0          # one cluster: nothing crosses
    # the paper's own remedy: at 1000x compression the same exchange hides behind 125 steps
    assert planner.comm_seconds(payload / 1000 * 4, 3, 1e9) < 125 * 1.0 * 3600


def test_overlap_plan_is_the_largest_rank_that_hides():
    from oracle import planner
    shapes = [(8192, 8192), (8192, 1024), (8192, 28672), (28672, 8192)]
    args = dict(qbits=4, group=128, extra_bytes=0, rmin=4, rmax=256, clusters=3,
                bits_per_second=1e9)
    r, H, t = planner.plan_overlap(shapes, step_seconds=0.05, H=1, **args)
    assert H == 1 and 4 <= r < 256 and t <= 0.05
    # one rank more would not fit
    over = planner.comm_seconds(planner.stage_payload_bytes(shapes, r + 1, 4, 128), 3, 1e9)
    assert over > 0.05
    # payload is monotone in r, so a longer budget never lowers the rank
    r2, _, _ = planner.plan_overlap(shapes, step_seconds=0.05, H=2, **args)
    assert r2 > r
    # nothing fits: rmin and the smallest H that hides it
    r3, H3, t3 = planner.plan_overlap(shapes, step_seconds=1e-3, H=1, **args)
    assert r3 == 4 and (H3 - 1) * 1e-3 < t3 <= H3 * 1e-3
    # two power iterations per round send every factor twice: the rank that hides is the one a
    # single iteration would get from half the budget (no other payload here)
    r_it2, _, t_it2 = planner.plan_overlap(shapes, step_seconds=0.05, H=2, iters=2, **args)
    assert r_it2 == r and abs(t_it2 - 2 * t) < 1e-12
    # factor payload accounting against the transmitted-factors reading (r = 2048 is about 2x)
    full = 8192 * 8192 * 2                       # FP16 bytes of one 8192 x 8192 matrix
    fac = planner.factor_payload_bytes(8192, 8192, 2048, 8, 128)
    assert 0.5 < fac / full * 2 < 0.52           # int8 codes: half the elements, one byte each


# --------------------------------------------------------------------------- exact pipeline
@pytest.mark.parametrize("qbits,K", [(8, 1), (8, 3), (4, 2)])
def test_quantised_lowrank_pipeline_is_exact_on_representable_input(qbits, K):
    # The decompressed average WITH the quantiser on, against a closed form: on this input the
    # whole of Alg. 1 (low-rank factors, both quantisations) and the AllReduce mean of Alg. 2 are
    # exact, so Delta equals the pseudo-gradient, the error buffers come out zero and the second
    # outer step moves theta by the Nesterov step of exactly that gradient.
    qmax = 2 ** (qbits - 1) - 1
    m, n, r, theta0, tl, q_in, delta = synth.exact_lowrank_case(qmax, K)
    orc = pipeline.MatrixOracle(theta0, K, q_in, qbits, 16, lr=0.5, mu=0.0)
    p_hat, q_bar = orc.step(tl)
    assert np.array_equal(orc.trace["delta"][0], delta)
    assert np.array_equal(np.abs(p_hat), np.full((r, m), 0.25, np.float32))
    assert np.array_equal(orc.delta_hat(), delta)
    codes = ref.unpack_codes(orc.trace["P_codes"][0], r * m, qbits)
    assert np.all(np.abs(codes) == qmax)                      # every entry sits on +-amax
    orc.set_basis(q_bar)
    orc.step([theta0.copy() for _ in range(K)])               # replicas did not move
    assert np.array_equal(orc.trace["e"][0], np.zeros((m, n), np.float32))
    assert np.array_equal(orc.theta, (-0.5 * delta).astype(np.float32))


# ---------------------------------------------------------------------------
# warm start across a rank change (Alg. 3 resizes the basis between two rounds)
# ---------------------------------------------------------------------------
def test_next_basis_hand_values_shrink_grow_same():
    q_bar = np.array([[1, 2], [3, 4], [5, 6]], np.float32)            # r_old = 3 columns, n = 2
    fresh = np.array([[7, 8], [9, 10], [11, 12]], np.float32)
    # shrink: the FIRST columns survive, in order; nothing of `fresh` is used
    assert pipeline.next_basis(q_bar, 2, fresh).tolist() == [[1, 2], [3, 4]]
    assert pipeline.next_basis(q_bar, 1, None).tolist() == [[1, 2]]
    # same rank: the basis itself (a copy, not a view of the oracle's state)
    same = pipeline.next_basis(q_bar, 3, fresh)
    assert same.tolist() == q_bar.tolist() and same is not q_bar and same.dtype == np.float32
    # grow: all old columns first, then the first r_new - r_old fresh columns, in order
    assert pipeline.next_basis(q_bar, 5, fresh).tolist() == [[1, 2], [3, 4], [5, 6], [7, 8], [9, 10]]
    assert pipeline.next_basis(q_bar, 4, fresh).tolist() == [[1, 2], [3, 4], [5, 6], [7, 8]]


def test_rank_change_rounds_keep_the_leading_subspace_and_the_schedule():
    """Three rounds of the oracle with the rank going 6 -> 3 -> 5 on one worker's exactly
    rank-3 pseudo-gradient whose right singular vectors are the first basis columns.  What the
    mathematics fixes: a basis cut to the first 3 columns still spans the gradient's row space,
    so the round reproduces it exactly; grown back with arbitrary fresh columns it still does
    (the fresh directions only add zero components); and the feedback of every round uses the
    factors at the rank they were formed with (the error buffer stays at rounding level)."""
    rng = np.random.default_rng(11)
    m, n = 24, 32
    U = synth.orthonormal_columns(rng, m, 3)
    V = synth.orthonormal_columns(rng, n, 6)
    G = ((U * np.array([3.0, 2.0, 1.0])) @ V[:, :3].T)                 # rank 3
    theta0 = rng.standard_normal((m, n)).astype(np.float32)
    orc = pipeline.MatrixOracle(theta0, 1, V.T.astype(np.float32), None, 16)
    ranks = [6, 3, 5]
    for t, r in enumerate(ranks, start=1):
        assert orc.q_in.shape[0] == r
        tl = [(orc.theta.astype(np.float64) - G).astype(np.float32)]
        orc.step(tl)
        assert orc.p_hat.shape == (r, m) and orc.q_bar.shape == (r, n)
        want = orc.trace["delta"][0].astype(np.float64)
        assert np.linalg.norm(orc.delta_hat() - want) <= 2e-6 * np.linalg.norm(want), (t, r)
        if t < len(ranks):
            fresh = rng.standard_normal((8, n)).astype(np.float32)
            nb = pipeline.next_basis(orc.q_bar, ranks[t], fresh)
            keep = min(r, ranks[t])
            assert np.array_equal(nb[:keep], orc.q_bar[:keep])
            orc.set_basis(nb)
    # feedback at the old rank: e = delta - Delta_hat stayed at rounding level throughout
    assert np.abs(orc.trace["e"][0]).max() <= 1e-5
    assert orc.n_applied == len(ranks) - 1


def test_oracle_resume_two_plus_one_equals_three_rounds():
    """The outer state is {theta, v, e_i, P_hat, Q_bar, basis, t}: three rounds in one object
    equal two rounds, the state copied into a new object, and the third round there."""
    m, n, K, r = 48, 64, 2, 6
    inp = synth.MatrixInputs(m, n, K, r, seed=31, sigma=1e-3, alpha=1.0)

    def tl(t):
        return [inp.theta_local(inp.theta_g, t, i) for i in range(K)]

    a = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, 4, 16)
    for t in (1, 2, 3):
        a.step(tl(t))
        a.set_basis(a.q_bar)
    b = pipeline.MatrixOracle(inp.theta_g, K, inp.q_in, 4, 16)
    for t in (1, 2):
        b.step(tl(t))
        b.set_basis(b.q_bar)
    c = pipeline.MatrixOracle(b.theta.copy(), K, b.q_in.copy(), 4, 16)
    c.v, c.ef = b.v.copy(), [e.copy() for e in b.ef]
    c.p_hat, c.q_bar, c.t, c.n_applied = b.p_hat.copy(), b.q_bar.copy(), b.t, b.n_applied
    c.step(tl(3))
    assert np.array_equal(c.theta, a.theta) and np.array_equal(c.v, a.v)
    assert np.array_equal(c.q_bar, a.q_bar) and np.array_equal(c.p_hat, a.p_hat)
    assert all(np.array_equal(x, y) for x, y in zip(c.ef, a.ef))
    assert c.n_applied == 2
