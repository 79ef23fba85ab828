// r' of Alg. 3 for one matrix: the smallest k whose k largest eigenvalues of S = Q_bar^T Q_bar
// hold at least tau of the trace (with P_hat orthonormal these are the squared singular values of
// the decompressed average).  S is accumulated in fp64 (same partial-sum kernel as the
// orthonormalisation); its eigenvalues come from a one-sided Jacobi iteration on the columns of S
// (S is symmetric positive semi-definite, so the column norms at convergence are the
// eigenvalues), run by one workgroup with a round-robin pair schedule; then sort, prefix sum and
// count, all in fp64.
#include "common.h"

namespace dlcx {

constexpr int kJT = 256;        // threads: 16 teams of 16 lanes, one column pair per team
constexpr int kMaxSweeps = 40;

__device__ __forceinline__ double team_sum(double v) {
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) v += __shfl_xor(v, off, 16);
    return v;
}

__global__ __launch_bounds__(kJT) void jacobi_rank_kernel(const double *__restrict__ part,
                                                          int nchunks, int r, double tau,
                                                          double *__restrict__ a_global,
                                                          int a_in_lds,
                                                          int32_t *__restrict__ rprime_out) {
    extern __shared__ double smem[];
    const int re = (r + 1) & ~1;                     // even number of columns (pad with zeros)
    double *a = a_in_lds ? smem : a_global;          // column-major re x re: a[col * re + row]
    __shared__ double eig[DLCX_MAX_RANK];
    __shared__ double sorted[DLCX_MAX_RANK];
    __shared__ int rotated;
    const int tid = threadIdx.x;
    for (int x = tid; x < re * re; x += kJT) {
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
            for (int pr = team; pr < npairs; pr += kJT / 16) {
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
    for (int c = tid; c < r; c += kJT) {
        double s = 0.0;
        for (int i = 0; i < re; ++i) s = fma(a[c * re + i], a[c * re + i], s);
        eig[c] = sqrt(s);
    }
    __syncthreads();
    for (int c = tid; c < r; c += kJT) {  // rank sort, descending, ties by index
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
    return (size_t)gram_chunks(L) * r * r * sizeof(double) + re * re * sizeof(double);
}

int launch_effective_rank(int64_t L, int r, const float *q_bar, double tau, int32_t *rprime_dev,
                          void *workspace, hipStream_t st) {
    double *part = reinterpret_cast<double *>(workspace);
    double *a = part + (size_t)gram_chunks(L) * r * r;
    int rc = launch_gram_partials(L, r, q_bar, part, st);
    if (rc != DLCX_OK) return rc;
    const size_t re = (size_t)((r + 1) & ~1);
    const size_t bytes = re * re * sizeof(double);
    const int in_lds = bytes <= 128 * 1024 ? 1 : 0;
    if (in_lds && bytes > 48 * 1024) {
        rc = note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(jacobi_rank_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes),
                      "jacobi attribute");
        if (rc != DLCX_OK) return rc;
    }
    Timed timed(KID_JACOBI, st);
    hipLaunchKernelGGL(jacobi_rank_kernel, dim3(1), dim3(kJT), in_lds ? bytes : 0, st, part,
                       gram_chunks(L), r, tau, a, in_lds, rprime_dev);
    return check_launch("jacobi_rank");
}

}  // namespace dlcx
