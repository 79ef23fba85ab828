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
    def __init__(self, theta_g, K, q_in, qbits, group, lr=0.7, mu=0.9):
        """qbits None switches the quantiser off (factors averaged exactly)."""
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
        # ---- Compressor, P phase
        self.trace["q_in"] = self.q_in.copy()
        P = [ref.project_p(self.ef[i], self.q_in) for i in range(self.K)]
        self.trace["P"] = P
        p_bar = self._avg(P, "P")
        self.trace["p_bar"] = p_bar
        self.p_hat = ref.orthonormalize(p_bar)
        # ---- Compressor, Q phase
        Q = [ref.project_q(self.ef[i], self.p_hat) for i in range(self.K)]
        self.trace["Q"] = Q
        self.q_bar = self._avg(Q, "Q")
        return self.p_hat, self.q_bar

    def delta_hat(self):
        return ref.reconstruct(self.p_hat, self.q_bar)

    def set_basis(self, q_in):
        self.q_in = np.ascontiguousarray(q_in, np.float32).copy()


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
