"""Call sequence of one outer step (Alg. 2) for the matrices of a pipeline stage.

Only sequencing lives here: which entry point of the HIP library runs on which buffers, in the
order of Alg. 2 with the one-step delay.  Every arithmetic step is a kernel of libdlcx_hip.so.

    t >= 2 :  e_i <- delta_i - Delta_hat^{t-1}                 dlcx_decompress
              delta_i <- (theta_g - theta_l,i) + e_i            dlcx_delta_ef
    t >= 2 :  theta_g <- OuterOpt(theta_g, Delta_hat^{t-1})     dlcx_outer_nesterov
              P phase: compress, average (+ orthonormalise)     dlcx_compress_batched, dlcx_average
              Q phase: compress, average                        dlcx_compress_batched, dlcx_average
"""
import ctypes as C

import torch

from . import (PHASE_P, PHASE_Q, desc, dlcx_average, dlcx_compress_batched, dlcx_decompress,
               dlcx_delta_ef, dlcx_ef_delta_apply, dlcx_outer_nesterov, dlcx_payload_bytes, dlcx_select_rank,
               dlcx_select_rank_workspace_bytes, dlcx_workspace_bytes)


class MatrixState:
    """Device buffers of one weight matrix: outer state, K error buffers, factors, payloads."""

    def __init__(self, theta_g, K, q_in, qbits, group, mma, r_max=None):
        self.m, self.n = theta_g.shape
        self.K, self.qbits, self.group, self.mma = K, qbits, group, mma
        dev = theta_g.device
        self.theta_g = theta_g
        self.v = torch.zeros_like(theta_g)
        self.ef = [torch.zeros_like(theta_g) for _ in range(K)]
        self.r = q_in.shape[0]
        self.r_max = r_max or self.r
        self.q_in = torch.empty(self.r_max, self.n, device=dev, dtype=torch.float32)
        self.q_in[: self.r].copy_(q_in)
        self.p_hat = torch.empty(self.r_max, self.m, device=dev, dtype=torch.float32)
        self.q_bar = torch.empty(self.r_max, self.n, device=dev, dtype=torch.float32)
        self.r_prev = 0  # rank of the factors held in p_hat / q_bar (0: none yet)
        dmax = desc(self.m, self.n, self.r_max, qbits, group, mma)
        _, cbp, sbp = dlcx_payload_bytes(dmax, PHASE_P)
        _, cbq, sbq = dlcx_payload_bytes(dmax, PHASE_Q)
        self.codes_p = [torch.empty(cbp, device=dev, dtype=torch.uint8) for _ in range(K)]
        self.scales_p = [torch.empty(sbp // 4, device=dev, dtype=torch.float32) for _ in range(K)]
        self.codes_q = [torch.empty(cbq, device=dev, dtype=torch.uint8) for _ in range(K)]
        self.scales_q = [torch.empty(sbq // 4, device=dev, dtype=torch.float32) for _ in range(K)]
        self.workspace_bytes = dlcx_workspace_bytes(dmax, K)

    def desc(self, r=None):
        return desc(self.m, self.n, self.r if r is None else r, self.qbits, self.group, self.mma)


class Stage:
    """All matrices of one pipeline stage plus shared scratch; `step` is one outer step.

    fused=True uses dlcx_ef_delta_apply (one pass for error buffers, pseudo-gradients and the
    outer update, the decompressed average never written); fused=False runs the separate entry
    points.  warm_start=True takes Q_bar of the previous round as the basis of the P phase.
    """

    def __init__(self, matrices, lr, mu, fused=False, warm_start=False):
        self.mats = matrices
        self.lr, self.mu = lr, mu
        self.fused, self.warm_start = fused, warm_start
        self.t = 0
        dev = matrices[0].theta_g.device
        ws = max(m.workspace_bytes for m in matrices)
        self.workspace = torch.empty(ws, device=dev, dtype=torch.uint8)
        self.delta_hat = None
        if not fused:
            big = max(m.m * m.n for m in matrices)
            self.delta_hat = torch.empty(big, device=dev, dtype=torch.float32)

    def params(self):
        return sum(m.m * m.n for m in self.mats)

    def step_matrix(self, M, theta_l, stream=None):
        t = self.t
        if t >= 2 and self.fused:
            dlcx_ef_delta_apply(M.desc(M.r_prev), M.p_hat, M.q_bar, theta_l, M.ef, M.theta_g, M.v,
                                self.lr, self.mu, workspace=self.workspace, stream=stream)
        else:
            if t >= 2:
                dlcx_decompress(M.desc(M.r_prev), M.p_hat, M.q_bar, self.delta_hat, M.ef,
                                workspace=self.workspace, stream=stream)
            for i in range(M.K):
                dlcx_delta_ef(M.theta_g, theta_l[i], M.ef[i], stream=stream)
            if t >= 2:
                dlcx_outer_nesterov(M.theta_g, M.v, self.delta_hat, self.lr, self.mu,
                                    numel=M.m * M.n, stream=stream)
        d = M.desc()
        basis = M.q_bar if (self.warm_start and t >= 2 and M.r_prev == M.r) else M.q_in
        dlcx_compress_batched(d, PHASE_P, M.ef, basis, M.codes_p, M.scales_p, self.workspace,
                              stream=stream)
        dlcx_average(d, PHASE_P, M.codes_p, M.scales_p, M.p_hat, self.workspace, stream=stream)
        dlcx_compress_batched(d, PHASE_Q, M.ef, M.p_hat, M.codes_q, M.scales_q, self.workspace,
                              stream=stream)
        dlcx_average(d, PHASE_Q, M.codes_q, M.scales_q, M.q_bar, self.workspace, stream=stream)
        M.r_prev = M.r

    def step(self, theta_l_per_matrix, stream=None):
        """theta_l_per_matrix[a][i]: local replica i of matrix a after this round's inner steps."""
        self.t += 1
        for M, tl in zip(self.mats, theta_l_per_matrix):
            self.step_matrix(M, tl, stream=stream)


class RankSelector:
    """Alg. 3 for a stage: measures r' on the latest Q_bar of every matrix, keeps the window."""

    def __init__(self, stage, c, r1, rmin, rmax, H1, tau=0.99):
        self.stage, self.c, self.r1, self.rmin, self.rmax, self.H1, self.tau = \
            stage, c, r1, rmin, rmax, H1, tau
        self.hist = (C.c_int32 * c)()
        descs = [M.desc(M.r_max) for M in stage.mats]
        nbytes = dlcx_select_rank_workspace_bytes(descs)
        self.workspace = torch.empty(nbytes, device=stage.mats[0].theta_g.device,
                                     dtype=torch.uint8)

    def first(self):
        """t = 1: r'_1 is defined as r_1."""
        return dlcx_select_rank([], [], self.tau, self.hist, 1, self.c, self.r1, self.rmin,
                                self.rmax, self.H1, rprime=self.r1)

    def next(self, t, stream=None):
        """Rank for outer step t >= 2 from the averages of step t-1."""
        descs = [M.desc(M.r_prev) for M in self.stage.mats]
        q_bars = [M.q_bar for M in self.stage.mats]
        return dlcx_select_rank(descs, q_bars, self.tau, self.hist, t, self.c, self.r1,
                                self.rmin, self.rmax, self.H1, workspace=self.workspace,
                                stream=stream)
