"""Call sequence of one outer step (Alg. 2) for the matrices of a pipeline stage.

Only sequencing lives here: which entry point of the HIP library runs on which buffers and on
which HIP stream, in the order of Alg. 2 with the one-step delay.  Every arithmetic step is a
kernel of libdlcx_hip.so.

    t >= 2 :  e_i <- delta_i - Delta_hat^{t-1}                 \\
              delta_i <- (theta_g - theta_l,i) + e_i            > dlcx_ef_delta_apply_compress, or
    t >= 2 :  theta_g <- OuterOpt(theta_g, Delta_hat^{t-1})    /  dlcx_decompress, dlcx_delta_ef,
                                                                  dlcx_outer_nesterov
              P phase: compress, average (+ orthonormalise)     dlcx_compress_batched, dlcx_average
              Q phase: compress, average                        dlcx_compress_batched, dlcx_average
              r' of the new average (Alg. 3)                    dlcx_effective_rank

The matrices of a stage are independent, so consecutive runs of them are dealt to a few HIP
streams (all at the default priority): the short, latency-bound kernels of one run (Cholesky,
Jacobi, quantiser; batched over the run) then go beside the HBM-bound sweeps of another.
"""
import ctypes as C

import torch

from . import (PHASE_P, PHASE_Q, desc, dlcx_average, dlcx_batched_workspace_bytes,
               dlcx_compress_batched, dlcx_decompress, dlcx_delta_ef, dlcx_dequant_average,
               dlcx_effective_rank, dlcx_effective_rank_batched, dlcx_ef_delta_apply_compress,
               dlcx_orthonormalize, dlcx_orthonormalize_batched, dlcx_outer_nesterov,
               dlcx_payload_bytes, dlcx_requantize, dlcx_select_rank_from, dlcx_workspace_bytes)


def plan_lanes(sizes, nstreams, chunk=0):
    """Deal matrices (element counts `sizes`, in order) to `nstreams` streams and cut every
    stream's share into batches.  Returns (lane_of, lane_chunks): lane_of[a] is the stream of
    matrix a -- consecutive runs with about the same number of elements each, by the position of
    a matrix's midpoint in the running total -- and lane_chunks[l] the list of half-open index
    ranges stream l works through: batches of `chunk` matrices (0: the length of the run), the
    first one cut to (l + 1) / nstreams of that, so that the streams are in different phases of
    the step (one in its projections while another is in its sweeps)."""
    total, acc, lane_of = sum(sizes), 0, []
    for size in sizes:
        mid = acc + size // 2
        lane_of.append(min(nstreams - 1, mid * nstreams // max(total, 1)))
        acc += size
    lane_chunks = []
    for lane in range(nstreams):
        idx = [a for a, l in enumerate(lane_of) if l == lane]
        lo, hi = (idx[0], idx[-1] + 1) if idx else (0, 0)
        chunks, a = [], lo
        size = chunk if chunk > 0 else max(hi - lo, 1)
        first = max(1, size * (lane + 1) // nstreams)
        while a < hi:
            b = min(hi, a + (first if not chunks else size))
            chunks.append((a, b))
            a = b
        lane_chunks.append(chunks)
    return lane_of, lane_chunks


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

    fused=True uses dlcx_ef_delta_apply_compress (one pass for error buffers, pseudo-gradients,
    outer update and the P-phase projection, the decompressed average never written);
    fused=False runs the separate entry points.  warm_start=True takes Q_bar of the previous
    round as the basis of the P phase.  streams > 1 deals consecutive runs of matrices to that
    many HIP streams.  measure_rank=True also launches the effective-rank kernel of Alg. 3 for
    every matrix (results in self.rprime_dev).  batched=True orthonormalises (and measures) the
    matrices of a stream `chunk` at a time in one batch between the two compression phases
    instead of matrix by matrix (chunk = 0: a stream's whole run).  requant=True re-encodes every
    averaged factor to q bits (dlcx_requantize), as a reduction that carries q-bit values would
    deliver it, before it is used.  iters > 1 repeats the two compression phases on the round's
    pseudo-gradients, each repeat starting from the Q average just formed (more power iterations
    per round: a closer rank-r fit for two more averages each).  stream_pool hands in the HIP
    streams to use (at least `streams` of them) instead of creating them.
    """

    def __init__(self, matrices, lr, mu, fused=False, warm_start=False, streams=1,
                 measure_rank=False, tau=0.99, batched=True, requant=False, iters=1, chunk=0,
                 stream_pool=None):
        assert iters >= 1 and chunk >= 0
        self.mats = matrices
        self.requant = requant
        self.iters = iters
        self.lr, self.mu = lr, mu
        self.fused, self.warm_start = fused, warm_start
        self.measure_rank, self.tau = measure_rank, tau
        self.t = 0
        dev = matrices[0].theta_g.device
        self.nstreams = max(1, min(streams, len(matrices)))
        ws = max(m.workspace_bytes for m in matrices)
        big = max(m.m * m.n for m in matrices)
        self.workspaces = [torch.empty(ws, device=dev, dtype=torch.uint8)
                           for _ in range(self.nstreams)]
        self.workspace = self.workspaces[0]
        self.delta_hats = [None] * self.nstreams
        if not fused:
            self.delta_hats = [torch.empty(big, device=dev, dtype=torch.float32)
                               for _ in range(self.nstreams)]
        if stream_pool:
            # the caller's streams (e.g. created with a compute-unit mask), one per lane
            assert len(stream_pool) >= self.nstreams
            self.side = list(stream_pool[: self.nstreams])
        else:
            self.side = [torch.cuda.Stream(device=dev) for _ in range(self.nstreams)] \
                if self.nstreams > 1 else []
        self.rprime_dev = torch.zeros(len(matrices), device=dev, dtype=torch.int32)
        self.batched = batched
        self.serial = False
        self.lane_of, self.lane_chunks = plan_lanes([M.m * M.n for M in matrices],
                                                    self.nstreams, chunk)
        self.batch_ws = [None] * self.nstreams
        if batched:
            for lane, chunks in enumerate(self.lane_chunks):
                nbytes = max([dlcx_batched_workspace_bytes([M.desc(M.r_max) for M in matrices[a:b]])
                              for a, b in chunks] + [256])
                self.batch_ws[lane] = torch.empty(nbytes, device=dev, dtype=torch.uint8)

    def params(self):
        return sum(m.m * m.n for m in self.mats)

    def _begin_and_p_phase(self, a, theta_l, lane, stream, orthonormalize):
        """Everything of Alg. 2 between two compressions, then the P phase, for matrix a."""
        M, t = self.mats[a], self.t
        ws, d_hat, d = self.workspaces[lane], self.delta_hats[lane], M.desc()
        # warm start: Q_bar of the previous round; after a rank change its first M.r columns
        # (the caller has filled columns beyond the previous rank with fresh draws)
        basis = M.q_bar if (self.warm_start and t >= 2) else M.q_in
        if self.fused:
            dlcx_ef_delta_apply_compress(d, M.r_prev if t >= 2 else 0, M.p_hat, M.q_bar, theta_l,
                                         M.ef, M.theta_g, M.v, self.lr, self.mu, basis,
                                         M.codes_p, M.scales_p, ws, stream=stream)
        else:
            if t >= 2:
                dlcx_decompress(M.desc(M.r_prev), M.p_hat, M.q_bar, d_hat, M.ef, workspace=ws,
                                stream=stream)
            for i in range(M.K):
                dlcx_delta_ef(M.theta_g, theta_l[i], M.ef[i], stream=stream)
            if t >= 2:
                dlcx_outer_nesterov(M.theta_g, M.v, d_hat, self.lr, self.mu, numel=M.m * M.n,
                                    stream=stream)
            dlcx_compress_batched(d, PHASE_P, M.ef, basis, M.codes_p, M.scales_p, ws,
                                  stream=stream)
        self._p_average(M, ws, stream, orthonormalize)

    def _p_phase_again(self, a, lane, stream, orthonormalize):
        """P phase of a further power iteration: basis = the Q average just formed."""
        M = self.mats[a]
        ws = self.workspaces[lane]
        dlcx_compress_batched(M.desc(), PHASE_P, M.ef, M.q_bar, M.codes_p, M.scales_p, ws,
                              stream=stream)
        self._p_average(M, ws, stream, orthonormalize)

    def _p_average(self, M, ws, stream, orthonormalize):
        d = M.desc()
        if orthonormalize and not self.requant:
            dlcx_average(d, PHASE_P, M.codes_p, M.scales_p, M.p_hat, ws, stream=stream)
            return
        # mean only; orthonormalised below, or by the stage in one batch afterwards
        dlcx_dequant_average(M.codes_p, M.scales_p, M.r * M.m, M.qbits, M.group, M.p_hat,
                             stream=stream)
        if self.requant:
            dlcx_requantize(M.p_hat, M.r * M.m, M.qbits, M.group, stream=stream)
        if orthonormalize:
            dlcx_orthonormalize(M.m, M.r, M.p_hat, ws, stream=stream)

    def _q_phase(self, a, lane, stream, rank):
        M = self.mats[a]
        ws, d = self.workspaces[lane], M.desc()
        dlcx_compress_batched(d, PHASE_Q, M.ef, M.p_hat, M.codes_q, M.scales_q, ws, stream=stream)
        dlcx_average(d, PHASE_Q, M.codes_q, M.scales_q, M.q_bar, ws, stream=stream)
        if self.requant:
            dlcx_requantize(M.q_bar, M.r * M.n, M.qbits, M.group, stream=stream)
        M.r_prev = M.r
        if rank:
            dlcx_effective_rank(M.n, M.r, M.q_bar, self.tau, self.rprime_dev[a:], ws,
                                stream=stream)

    def _fork(self):
        if not self.side or self.serial:
            return None
        main = torch.cuda.current_stream()
        start = torch.cuda.Event()
        start.record(main)
        for s in self.side:
            s.wait_event(start)
        return main

    def _join(self, main):
        if main is None:
            return
        for s in self.side:
            done = torch.cuda.Event()
            done.record(s)
            main.wait_event(done)

    def _lane(self, a):
        if self.serial:
            return 0, None
        lane = self.lane_of[a]
        return lane, (self.side[lane] if self.side else None)

    def step(self, theta_l_per_matrix, serial=False):
        """theta_l_per_matrix[a][i]: local replica i of matrix a after this round's inner steps.
        Work is issued on the current stream (and the side streams, joined before returning);
        serial=True keeps everything on the current stream (kernels then run one at a time)."""
        self.t += 1
        self.serial = serial
        n = len(self.mats)
        if not self.batched:
            main = self._fork()
            for a in range(n):
                lane, st = self._lane(a)
                self._begin_and_p_phase(a, theta_l_per_matrix[a], lane, st, orthonormalize=True)
                for j in range(1, self.iters):
                    self._q_phase(a, lane, st, rank=False)
                    self._p_phase_again(a, lane, st, orthonormalize=True)
                self._q_phase(a, lane, st, rank=self.measure_rank)
            self._join(main)
            return
        # each lane batches its own matrices: the latency-bound batched kernels of one lane run
        # beside the HBM-bound sweeps of the others, and no lane waits for another inside a step
        main = self._fork()
        # batches are issued round-robin over the lanes (each lane's own in order), so that every
        # stream has work queued from the start of the step
        order = [(lane, chunks[c]) for c in range(max(len(x) for x in self.lane_chunks))
                 for lane, chunks in enumerate(self.lane_chunks) if c < len(chunks)]
        for lane, (lo, hi) in order:
            _, st = self._lane(lo)
            mats = self.mats[lo:hi]
            descs = [M.desc() for M in mats]
            for j in range(self.iters):
                for a in range(lo, hi):
                    if j == 0:
                        self._begin_and_p_phase(a, theta_l_per_matrix[a], lane, st,
                                                orthonormalize=False)
                    else:
                        self._p_phase_again(a, lane, st, orthonormalize=False)
                dlcx_orthonormalize_batched(descs, [M.p_hat for M in mats],
                                            self.batch_ws[lane], stream=st)
                for a in range(lo, hi):
                    self._q_phase(a, lane, st, rank=False)
            if self.measure_rank:
                dlcx_effective_rank_batched(descs, [M.q_bar for M in mats], self.tau,
                                            self.rprime_dev[lo:], self.batch_ws[lane],
                                            stream=st)
        self._join(main)


    def set_rank(self, r_next, fresh=None):
        """Rank of the next compression (Alg. 3's r_t) for every matrix of the stage, with the
        warm start resized to it: the first min(r_old, r_next) columns of the basis stay where
        they are, and when the rank grows, columns r_old .. r_next - 1 of matrix a are copied
        from fresh[a] (a device tensor with at least r_next - r_old rows of length n; the draws
        are the caller's, nothing is generated here).  The basis is Q_bar of the round just
        finished when the stage warm-starts and a round has run, else Q_in.  A matrix's rank is
        clipped to its smaller side and to the capacity its buffers were allocated for.  The
        previous round's factors (and their rank) are untouched: the next step still feeds back
        and applies the average at the rank it was formed with."""
        for a, M in enumerate(self.mats):
            r_new = max(1, min(r_next, M.r_max, M.m, M.n))
            grow = r_new - M.r
            if grow > 0:
                assert fresh is not None and fresh[a].shape[0] >= grow and fresh[a].shape[1] == M.n
                basis = M.q_bar if (self.warm_start and self.t >= 1) else M.q_in
                basis[M.r:r_new].copy_(fresh[a][:grow])
            M.r = r_new

    def capture(self, theta_l_per_matrix):
        """Record one outer step into a HIP graph (every launch of `step`, on all its streams)
        and return it; `replay` then issues the whole step with one call.  Call after at least
        two eager steps, so that the recorded step is the steady one (feedback and update from
        a previous average) and every kernel has been launched once; the ranks and the buffers
        (theta_l included) are those of the recording.  Nothing runs while recording."""
        assert self.t >= 2
        t_before = self.t
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step(theta_l_per_matrix)
        self.t = t_before
        self.graph = graph
        return graph

    def replay(self):
        self.t += 1
        self.graph.replay()


class RankSelector:
    """Alg. 3 for a stage: window rule over the r' values the stage measured (measure_rank)."""

    def __init__(self, stage, c, r1, rmin, rmax, H1):
        self.stage, self.c, self.r1, self.rmin, self.rmax, self.H1 = stage, c, r1, rmin, rmax, H1
        self.hist = (C.c_int32 * c)()

    def first(self):
        """t = 1: r'_1 is defined as r_1."""
        return dlcx_select_rank_from(None, 0, self.hist, 1, self.c, self.r1, self.rmin, self.rmax,
                                     self.H1, rprime=self.r1)

    def next(self, t):
        """Rank for outer step t >= 2 from the averages of step t-1 (synchronises)."""
        return dlcx_select_rank_from(self.stage.rprime_dev, len(self.stage.mats), self.hist, t,
                                     self.c, self.r1, self.rmin, self.rmax, self.H1)
