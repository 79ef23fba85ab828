// r' of Alg. 3 for one matrix: the smallest k whose k largest eigenvalues of S = Q_bar^T Q_bar
// hold at least tau of the trace (with P_hat orthonormal these are the squared singular values of
// the decompressed average).  S is accumulated in fp64 (same partial-sum kernel as the
// orthonormalisation).  One workgroup per matrix finds its eigenvalues, all in fp64:
//   r  < 32:  one-sided Jacobi iteration on the columns of S in LDS (S is symmetric positive
//             semi-definite, so the column norms at convergence are the eigenvalues) with a
//             round-robin pair schedule;
//   r >= 32:  Householder reduction to tridiagonal form (each step one symmetric matrix-vector
//             product and one rank-2 update of the trailing block; S in LDS up to r = 128, in
//             global memory / L2 above), then every eigenvalue by bisection on the Sturm
//             sequence, one thread each.  (Measured per batch of 12: r = 64 1.56 -> 0.55 ms,
//             r = 128 9.6 -> 1.6 ms against the Jacobi route; r = 16 the same.)
// Then sort, prefix sum and count.
#include "common.h"

namespace dlcx {

constexpr int kJT = 1024;       // at most 64 teams of 16 lanes, one column pair per team
constexpr int kMaxSweeps = 40;

__device__ __forceinline__ double team_sum(double v) {
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) v += __shfl_xor(v, off, 16);
    return v;
}

constexpr size_t kJacobiLdsMax = 128 * 1024;
constexpr int kTriMinRank = 32;  // from here on the tridiagonal route is the faster one

// Sum of one value per thread over the workgroup, in a fixed order; every thread gets it.
__device__ __forceinline__ double block_sum(double v, double *red, int nthreads) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    __syncthreads();  // earlier readers of red are done
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < nthreads / 64; ++w) s += red[w];
    return s;
}

// Eigenvalues of the symmetric r x r matrix a (column-major, leading dimension ld, both halves
// stored, in LDS or global memory), descending, negative ones clamped to zero, into out[0..r).
// d, e, v, w: r doubles each; psum: (nthreads / 256) * 256 doubles; red: 16 doubles (all LDS).
__device__ void tridiagonal_eigenvalues(double *a, int r, int ld, double *d, double *e, double *v,
                                        double *w, double *psum, double *red, double *out,
                                        int nthreads) {
    const int tid = threadIdx.x;
    const int parts = nthreads / 256;
    for (int k = 0; k + 2 < r; ++k) {
        const int L = r - k - 1;
        double *x = a + (int64_t)k * ld + k + 1;  // column k below the diagonal
        const double xt = tid < L ? x[tid] : 0.0;
        const double sumsq = block_sum(xt * xt, red, nthreads);
        const double x0 = x[0];
        const double tail = sumsq - x0 * x0;
        if (tid == 0) d[k] = a[(int64_t)k * ld + k];
        if (!(tail > 0.0)) {  // already tridiagonal in this column: no reflection
            if (tid == 0) e[k] = x0;
            __syncthreads();
            continue;
        }
        const double alpha = -copysign(sqrt(sumsq), x0);
        const double v0 = x0 - alpha;
        const double beta = 2.0 / (tail + v0 * v0);
        if (tid < L) v[tid] = tid == 0 ? v0 : xt;
        if (tid == 0) e[k] = alpha;
        __syncthreads();
        // p = beta * A22 v: thread (part, i) sums its quarter of the columns of row i
        double *a22 = a + (int64_t)(k + 1) * ld + k + 1;
        {
            const int i = tid & 255, part = tid >> 8;
            const int per = (L + parts - 1) / parts;
            const int j0 = part * per, j1 = j0 + per < L ? j0 + per : L;
            double acc = 0.0;
            if (i < L)
                for (int j = j0; j < j1; ++j) acc = fma(a22[(int64_t)j * ld + i], v[j], acc);
            psum[part * 256 + i] = acc;
        }
        __syncthreads();
        double pi = 0.0;
        if (tid < L) {
            for (int q = 0; q < parts; ++q) pi += psum[q * 256 + tid];
            pi *= beta;
        }
        const double vp = block_sum(tid < L ? v[tid] * pi : 0.0, red, nthreads);
        const double kk = 0.5 * beta * vp;
        if (tid < L) w[tid] = pi - kk * v[tid];
        __syncthreads();
        // A22 <- A22 - v w^T - w v^T
        for (int idx = tid; idx < L * L; idx += nthreads) {
            const int i = idx % L, j = idx / L;
            double *p = a22 + (int64_t)j * ld + i;
            *p = *p - (v[i] * w[j] + w[i] * v[j]);
        }
        __threadfence_block();
        __syncthreads();
    }
    if (tid == 0) {
        if (r >= 2) {
            d[r - 2] = a[(int64_t)(r - 2) * ld + r - 2];
            e[r - 2] = a[(int64_t)(r - 2) * ld + r - 1];
        }
        d[r - 1] = a[(int64_t)(r - 1) * ld + r - 1];
    }
    __syncthreads();
    // Gershgorin interval, then the c-th largest eigenvalue by bisection: the number of negative
    // terms of the Sturm sequence at x is the number of eigenvalues below x
    double lo0 = d[0], hi0 = d[0];
    for (int i = 0; i < r; ++i) {
        const double rad = (i > 0 ? fabs(e[i - 1]) : 0.0) + (i + 1 < r ? fabs(e[i]) : 0.0);
        lo0 = fmin(lo0, d[i] - rad);
        hi0 = fmax(hi0, d[i] + rad);
    }
    for (int c = tid; c < r; c += nthreads) {
        const int below = r - 1 - c;  // eigenvalues smaller than the one wanted
        double lo = lo0, hi = hi0;
        for (int itn = 0; itn < 200; ++itn) {
            const double mid = 0.5 * (lo + hi);
            if (!(mid > lo && mid < hi)) break;
            int cnt = 0;
            double q = d[0] - mid;
            cnt += q < 0.0;
            for (int i = 1; i < r; ++i) {
                if (fabs(q) < 1e-300) q = -1e-300;
                q = d[i] - mid - e[i - 1] * e[i - 1] / q;
                cnt += q < 0.0;
            }
            if (cnt > below) hi = mid;
            else lo = mid;
        }
        out[c] = fmax(0.5 * (lo + hi), 0.0);
    }
    __syncthreads();
}

__global__ __launch_bounds__(kJT) void jacobi_rank_kernel(FactorBatch batch, double tau) {
    const int nthreads = blockDim.x;  // 256 .. 1024: one team of 16 lanes per column pair
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
    __shared__ double tri_e[DLCX_MAX_RANK], tri_v[DLCX_MAX_RANK], tri_w[DLCX_MAX_RANK];
    __shared__ double tri_psum[(kJT / 256) * 256], tri_red[kJT / 64];
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
    const bool tri = !a_in_lds || r >= kTriMinRank;
    if (tri) {
        __threadfence_block();
        tridiagonal_eigenvalues(a, r, re, eig, tri_e, tri_v, tri_w, tri_psum, tri_red, sorted,
                                nthreads);
    }
    for (int sweep = 0; !tri && sweep < kMaxSweeps; ++sweep) {
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
    if (!tri) {
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
    }
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
    FactorBatch summed;  // the same factors with their Gram sums in one chunk
    int rc = launch_gram_partials_batch(batch, &summed, st);
    if (rc != DLCX_OK) return rc;
    size_t bytes = 0;
    for (int i = 0; i < batch.n; ++i) {
        const size_t re = (size_t)((batch.it[i].r + 1) & ~1);
        const size_t b = re * re * sizeof(double);
        if (b <= kJacobiLdsMax && b > bytes) bytes = b;
    }
    static size_t granted = 0;
    rc = grant_dynamic_lds(reinterpret_cast<const void *>(jacobi_rank_kernel), bytes, &granted,
                           "jacobi attribute");
    if (rc != DLCX_OK) return rc;
    Timed timed(KID_JACOBI, st);
    int rmax = 0;
    for (int i = 0; i < batch.n; ++i) rmax = batch.it[i].r > rmax ? batch.it[i].r : rmax;
    // a team of 16 lanes per column pair of the largest matrix (r / 2 pairs), so that a step of
    // the pair schedule is one pass; 1024 threads for the tridiagonal path
    int threads = ((rmax + 1) / 2 * 16 + 255) / 256 * 256;
    threads = threads < 256 ? 256 : (threads > kJT || rmax > 128 ? kJT : threads);
    hipLaunchKernelGGL(jacobi_rank_kernel, dim3((unsigned)batch.n), dim3((unsigned)threads), bytes,
                       st, summed, tau);
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
