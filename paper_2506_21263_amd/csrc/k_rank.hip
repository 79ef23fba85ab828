// r' of Alg. 3 for one matrix: the smallest k whose k largest eigenvalues of S = Q_bar^T Q_bar
// hold at least tau of the trace (with P_hat orthonormal these are the squared singular values of
// the decompressed average).  S is accumulated in fp64 (same partial-sum kernel as the
// orthonormalisation); its eigenvalues come from a one-sided Jacobi iteration on the columns of S
// (S is symmetric positive semi-definite, so the column norms at convergence are the
// eigenvalues), run by one workgroup with a round-robin pair schedule; then sort, prefix sum and
// count, all in fp64.
#include "common.h"

namespace dlcx {

constexpr int kJT = 1024;       // at most 64 teams of 16 lanes, one column pair per team
constexpr int kMaxSweeps = 40;

__device__ __forceinline__ double team_sum(double v) {
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) v += __shfl_xor(v, off, 16);
    return v;
}

constexpr size_t kJacobiLdsMax = 140 * 1024;

__global__ __launch_bounds__(kJT) void jacobi_rank_kernel(FactorBatch batch, double tau) {
    const int nthreads = blockDim.x;  // 256 for small matrices, 1024 when r > 128
    extern __shared__ double smem[];
    const FactorItem it = batch.it[blockIdx.x];
    const int r = it.r, nchunks = it.nchunks;
    const double *__restrict__ part = it.part;
    int32_t *__restrict__ rprime_out = it.out;
    const int re = (r + 1) & ~1;                     // even number of columns (pad with zeros)
    const bool a_in_lds = (size_t)re * re * sizeof(double) <= kJacobiLdsMax;
    double *a = a_in_lds ? smem : it.g;              // column-major re x re: a[col * re + row]
    __shared__ double eig[DLCX_MAX_RANK];
    __shared__ double sorted[DLCX_MAX_RANK];
    __shared__ int rotated;
    const int tid = threadIdx.x;
    for (int x = tid; x < re * re; x += nthreads) {
        const int col = x / re, row = x % re;
        double s = 0.0;
        if (col < r && row < r) {
            const int lo = row < col ? row : col, hi = row < col ? col : row;
            for (int c = 0; c < nchunks; ++c) s += part[(int64_t)c * r * r + lo * r + hi];
        }
        a[x] = s;
    }
    __syncthreads();
    const int team = tid >> 4, lane = tid & 15;
    const int npairs = re / 2;
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        if (tid == 0) rotated = 0;
        __syncthreads();
        for (int step = 0; step < re - 1; ++step) {
            for (int pr = team; pr < npairs; pr += nthreads / 16) {
                // round-robin tournament: pair 0 is (re-1, step); pair k is
                // ((step + k) mod (re-1), (step - k) mod (re-1))
                int p, q;
                if (pr == 0) {
                    p = re - 1;
                    q = step;
                } else {
                    p = (step + pr) % (re - 1);
                    q = (step - pr + (re - 1)) % (re - 1);
                }
                double *cp = a + p * re, *cq = a + q * re;
                double alpha = 0.0, beta = 0.0, gamma = 0.0;
                for (int i = lane; i < re; i += 16) {
                    const double x = cp[i], y = cq[i];
                    alpha = fma(x, x, alpha);
                    beta = fma(y, y, beta);
                    gamma = fma(x, y, gamma);
                }
                alpha = team_sum(alpha);
                beta = team_sum(beta);
                gamma = team_sum(gamma);
                if (gamma * gamma > 1e-26 * alpha * beta) {
                    const double zeta = (beta - alpha) / (2.0 * gamma);
                    const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    const double cs = 1.0 / sqrt(1.0 + t * t), sn = cs * t;
                    for (int i = lane; i < re; i += 16) {
                        const double x = cp[i], y = cq[i];
                        cp[i] = cs * x - sn * y;
                        cq[i] = sn * x + cs * y;
                    }
                    if (lane == 0) rotated = 1;
                }
            }
            __syncthreads();
        }
        const int any = rotated;
        __syncthreads();
        if (!any) break;
    }
    for (int c = tid; c < r; c += nthreads) {
        double s = 0.0;
        for (int i = 0; i < re; ++i) s = fma(a[c * re + i], a[c * re + i], s);
        eig[c] = sqrt(s);
    }
    __syncthreads();
    for (int c = tid; c < r; c += nthreads) {  // rank sort, descending, ties by index
        const double e = eig[c];
        int pos = 0;
        for (int u = 0; u < r; ++u) pos += (eig[u] > e) || (eig[u] == e && u < c);
        sorted[pos] = e;
    }
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
        for (int c = 0; c < r; ++c) total += sorted[c];
        int rp = 0;
        if (total > 0.0) {
            double cum = 0.0;
            rp = r;
            for (int c = 0; c < r; ++c) {
                cum += sorted[c];
                if (cum >= tau * total) {
                    rp = c + 1;
                    break;
                }
            }
        }
        *rprime_out = rp;
    }
}

size_t effrank_workspace_bytes(int64_t L, int r) {
    const size_t re = (size_t)((r + 1) & ~1);
    return a256x(((size_t)gram_chunks(L) * r * r + re * re) * sizeof(double));
}

void effrank_item(FactorItem *it, const float *q_bar, int64_t L, int r, int32_t *out,
                  void *workspace) {
    it->f = const_cast<float *>(q_bar);  // only read
    it->L = L;
    it->r = r;
    it->nchunks = gram_chunks(L);
    it->part = reinterpret_cast<double *>(workspace);
    it->g = it->part + (size_t)it->nchunks * r * r;
    it->w = nullptr;
    it->out = out;
}

int launch_effective_rank_batch(const FactorBatch &batch, double tau, hipStream_t st) {
    if (batch.n == 0) return DLCX_OK;
    int rc = launch_gram_partials_batch(batch, st);
    if (rc != DLCX_OK) return rc;
    size_t bytes = 0;
    for (int i = 0; i < batch.n; ++i) {
        const size_t re = (size_t)((batch.it[i].r + 1) & ~1);
        const size_t b = re * re * sizeof(double);
        if (b <= kJacobiLdsMax && b > bytes) bytes = b;
    }
    static size_t granted = 0;
    if (bytes > 48 * 1024 && bytes > granted) {
        rc = note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(jacobi_rank_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes),
                      "jacobi attribute");
        if (rc != DLCX_OK) return rc;
        granted = bytes;
    }
    Timed timed(KID_JACOBI, st);
    int rmax = 0;
    for (int i = 0; i < batch.n; ++i) rmax = batch.it[i].r > rmax ? batch.it[i].r : rmax;
    hipLaunchKernelGGL(jacobi_rank_kernel, dim3((unsigned)batch.n), dim3(rmax > 128 ? 1024 : 256),
                       bytes, st, batch, tau);
    return check_launch("jacobi_rank");
}

int launch_effective_rank(int64_t L, int r, const float *q_bar, double tau, int32_t *rprime_dev,
                          void *workspace, hipStream_t st) {
    FactorBatch b;
    b.n = 1;
    effrank_item(&b.it[0], q_bar, L, r, rprime_dev, workspace);
    return launch_effective_rank_batch(b, tau, st);
}

}  // namespace dlcx
