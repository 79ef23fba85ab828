"""The outer step of Alg. 2 for ONE weight matrix, written with the oracle's steps.

TEST INFRASTRUCTURE ONLY (see oracle/ref.py).

One call of `MatrixOracle.step` is outer step t of Alg. 2 for one pipeline
stage's matrix, with the D data-parallel workers simulated as K entries of a
list, in the order the algorithm prints them:

  t >= 2 :  e_i      <- delta_i^{t-1} - Delta^{t-1}            (error buffer)
            delta_i  <- (theta^{t-1} - theta_i^t) + e_i         (pseudo-gradient)
  t >= 2 :  theta^t  <- OuterOpt(theta^{t-1}, Delta^{t-1})      (one-step delay)
            Delta^t  <- mean_i C(delta_i^t | q, r)              (compress, "AllReduce")

where C is Alg. 1 read as one shared-basis subspace iteration whose factors are
quantised and averaged:  P_i = delta_i Q_in -> quantise -> mean -> orthonormalise
-> P_hat;  Q_i = delta_i^T P_hat -> quantise -> mean -> Q_bar;
Delta = P_hat Q_bar^T.  Nothing is applied at t = 1 and the last Delta is
produced but never applied, as in the paper.
"""
import numpy as np

from . import ref


def _mean64(factors):
    acc = np.zeros(factors[0].shape, np.float64)
    for f in factors:
        acc += f.astype(np.float64)
    return (acc / len(factors)).astype(np.float32)


class MatrixOracle:
    def __init__(self, theta_g, K, q_in, qbits, group, lr=0.7, mu=0.9, requant=False, iters=1):
        """qbits None switches the quantiser off (factors averaged exactly); requant re-encodes
        each averaged factor to q bits, as a low-bit reduction would hand it on; iters is the
        number of power iterations the LOWRANK step of Alg. 1 takes per round (1 in the paper;
        every further one is a P phase from the Q average just formed, then a Q phase, on the
        same pseudo-gradients -- subspace iteration, two more averages each)."""
        assert iters >= 1
        self.requant = requant
        self.iters = iters
        self.m, self.n = theta_g.shape
        self.K = K
        self.theta = np.ascontiguousarray(theta_g, np.float32).copy()
        self.v = np.zeros_like(self.theta)
        # e_i before delta_ef, delta_i after it: one buffer per worker, as in the library
        self.ef = [np.zeros_like(self.theta) for _ in range(K)]
        self.q_in = np.ascontiguousarray(q_in, np.float32).copy()
        self.qbits, self.group = qbits, group
        self.lr, self.mu = lr, mu
        self.p_hat = None
        self.q_bar = None
        self.t = 0
        self.n_applied = 0
        self.trace = {}

    def _avg(self, factors, tag):
        """quantise each worker's factor, then the in-order mean of the dequantised payloads."""
        if self.qbits is None:
            return _mean64(factors)
        codes, scales = [], []
        for f in factors:
            c, s = ref.quantize(f, self.qbits, self.group)
            codes.append(c)
            scales.append(s)
        self.trace[tag + "_codes"] = codes
        self.trace[tag + "_scales"] = scales
        flat = ref.dequant_average(codes, scales, factors[0].size, self.qbits, self.group)
        if self.requant:
            flat = requantize(flat, self.qbits, self.group)
        return flat.reshape(factors[0].shape)

    def step(self, theta_l):
        """theta_l: list of K local replicas after H inner steps (float32, or uint16 bf16 bits)."""
        self.t += 1
        self.trace = {}
        d_hat_prev = None
        if self.t >= 2:
            d_hat_prev = ref.reconstruct(self.p_hat, self.q_bar)
            self.trace["delta_hat_prev"] = d_hat_prev
            for i in range(self.K):
                ref.ef_update(self.ef[i].reshape(-1), d_hat_prev.reshape(-1))
            self.trace["e"] = [e.copy() for e in self.ef]
        for i in range(self.K):
            tl = np.ascontiguousarray(theta_l[i]).reshape(-1)
            self.ef[i] = ref.delta_ef(self.theta.reshape(-1), tl,
                                      self.ef[i].reshape(-1)).reshape(self.m, self.n)
        self.trace["delta"] = [d.copy() for d in self.ef]
        if self.t >= 2:
            ref.outer_nesterov(self.theta.reshape(-1), self.v.reshape(-1),
                               d_hat_prev.reshape(-1), self.lr, self.mu)
            self.n_applied += 1
        basis = self.q_in
        for j in range(self.iters):
            sfx = "" if j == 0 else "@%d" % j  # trace keys of the iterations after the first
            # ---- Compressor, P phase
            self.trace["q_in" + sfx] = basis.copy()
            P = [ref.project_p(self.ef[i], basis) for i in range(self.K)]
            self.trace["P" + sfx] = P
            p_bar = self._avg(P, "P" + sfx)
            self.trace["p_bar" + sfx] = p_bar
            self.p_hat = ref.orthonormalize(p_bar)
            self.trace["p_hat" + sfx] = self.p_hat
            # ---- Compressor, Q phase
            Q = [ref.project_q(self.ef[i], self.p_hat) for i in range(self.K)]
            self.trace["Q" + sfx] = Q
            self.q_bar = self._avg(Q, "Q" + sfx)
            self.trace["q_bar" + sfx] = self.q_bar
            basis = self.q_bar
        return self.p_hat, self.q_bar

    def delta_hat(self):
        return ref.reconstruct(self.p_hat, self.q_bar)

    def set_basis(self, q_in):
        self.q_in = np.ascontiguousarray(q_in, np.float32).copy()


class TensorOracle:
    """The outer step of Alg. 2 with the compressor reduced to its quantiser.

    Alg. 1 with the LOWRANK step left out, C(delta) = QUANTIZE(delta | q), is the setting the
    paper reports for its smaller model (Sec. 4.1: Int4 only, no rank adaptation) and the only
    one that applies to tensors that are not matrices (norm weights, biases).  The tensor is a
    flat array whose length is a multiple of the group size; groups are runs of `group`
    consecutive elements.  Same schedule as MatrixOracle:

      t >= 2 :  e_i      <- delta_i^{t-1} - Delta^{t-1}
                delta_i  <- (theta^{t-1} - theta_i^t) + e_i
      t >= 2 :  theta^t  <- OuterOpt(theta^{t-1}, Delta^{t-1})
                Delta^t  <- mean_i dequant(QUANTIZE(delta_i^t))   [re-encoded to q bits if requant]
    """

    def __init__(self, theta_g, K, qbits, group, lr=0.7, mu=0.9, requant=False):
        self.theta = np.ascontiguousarray(theta_g, np.float32).reshape(-1).copy()
        self.numel = self.theta.size
        assert self.numel % group == 0
        self.K, self.qbits, self.group = K, qbits, group
        self.lr, self.mu, self.requant = lr, mu, requant
        self.v = np.zeros_like(self.theta)
        self.ef = [np.zeros_like(self.theta) for _ in range(K)]
        self.codes, self.scales = None, None
        self.t = 0
        self.n_applied = 0
        self.trace = {}

    def delta_hat(self):
        """Delta of the last completed compression (what the next round applies and feeds back)."""
        mean = ref.dequant_average(self.codes, self.scales, self.numel, self.qbits, self.group)
        if self.requant:
            mean = requantize(mean, self.qbits, self.group)
        return mean

    def step(self, theta_l):
        self.t += 1
        self.trace = {}
        d_hat_prev = None
        if self.t >= 2:
            d_hat_prev = self.delta_hat()
            self.trace["delta_hat_prev"] = d_hat_prev
            for i in range(self.K):
                ref.ef_update(self.ef[i], d_hat_prev)
            self.trace["e"] = [e.copy() for e in self.ef]
        for i in range(self.K):
            tl = np.ascontiguousarray(theta_l[i]).reshape(-1)
            self.ef[i] = ref.delta_ef(self.theta, tl, self.ef[i])
        self.trace["delta"] = [d.copy() for d in self.ef]
        if self.t >= 2:
            ref.outer_nesterov(self.theta, self.v, d_hat_prev, self.lr, self.mu)
            self.n_applied += 1
        self.codes, self.scales = [], []
        for i in range(self.K):
            c, s = ref.quantize(self.ef[i], self.qbits, self.group)
            self.codes.append(c)
            self.scales.append(s)
        return self.codes, self.scales


def requantize(x, qbits, group):
    """A mean re-encoded to q bits, as a low-bit reduction would hand it on: the quantiser
    followed by its decoder."""
    shape = x.shape
    c, s = ref.quantize(np.ascontiguousarray(x, np.float32).reshape(-1), qbits, group)
    return ref.dequantize(c, s, x.size, qbits, group).reshape(shape)


def next_basis(q_bar, r_new, fresh):
    """Warm start: the first min(r_old, r_new) columns of Q_bar, then columns of `fresh`."""
    r_old, n = q_bar.shape
    out = np.empty((r_new, n), np.float32)
    keep = min(r_old, r_new)
    out[:keep] = q_bar[:keep]
    if r_new > keep:
        out[keep:] = fresh[: r_new - keep]
    return out


def stage_rprime(per_matrix_rprime, rmin):
    """Stage value of r': a zero-trace matrix counts as rmin, mean rounded half-up."""
    vals = [rp if rp > 0 else rmin for rp in per_matrix_rprime]
    s, k = sum(vals), len(vals)
    return (2 * s + k) // (2 * k)
