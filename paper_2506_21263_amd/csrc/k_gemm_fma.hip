// Rank-r products of the low-rank compressor on the vector ALU (DLCX_MMA_FMA): fp32 operands,
// fp64 accumulation.  This is the accuracy mode: it is not meant to reach the roofline, it is the
// GPU path whose rounding is closest to the exact products, and it accepts every shape the
// interface allows.  The MFMA modes live in k_gemm_mfma.hip.
#include <type_traits>

#include "common.h"

namespace dlcx {

constexpr int kT = 256;    // threads per workgroup
constexpr int kRows = 64;  // rows (P phase) or columns (Q phase) per workgroup
constexpr int kTk = 32;    // reduction chunk staged in LDS

// ---------------------------------------------------------------------------------------------
// P_k = delta_k * Q_in.  Workgroup: 64 rows of delta, all r outputs; wave w owns the outputs
// c = w, w+4, ...; lanes are rows, so the Q_in operand is a wave-uniform LDS broadcast.
// ---------------------------------------------------------------------------------------------
template <int kAcc>  // accumulators per thread, >= ceil(r / 4)
__global__ __launch_bounds__(kT) void project_p_fma_kernel(PtrPack<const float *> deltas,
                                                           const float *__restrict__ q_in,
                                                           PtrPack<float *> outs, int64_t m,
                                                           int64_t n, int r) {
    extern __shared__ float lds[];
    float *dl = lds;                        // [kRows][kTk + 1]
    float *ql = lds + kRows * (kTk + 1);    // [r][kTk + 1]
    const float *__restrict__ delta = deltas.p[blockIdx.y];
    float *__restrict__ out = outs.p[blockIdx.y];
    const int64_t i0 = (int64_t)blockIdx.x * kRows;
    const int lane_row = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    double acc[kAcc];
#pragma unroll
    for (int u = 0; u < kAcc; ++u) acc[u] = 0.0;

    for (int64_t j0 = 0; j0 < n; j0 += kTk) {
        for (int idx = threadIdx.x; idx < kRows * (kTk / 4); idx += kT) {
            const int row = idx / (kTk / 4), c4 = idx % (kTk / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + row < m && j0 + c4 * 4 < n)
                v = *reinterpret_cast<const float4 *>(delta + (i0 + row) * n + j0 + c4 * 4);
            float *d = dl + row * (kTk + 1) + c4 * 4;
            d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
        }
        for (int idx = threadIdx.x; idx < r * (kTk / 4); idx += kT) {
            const int c = idx / (kTk / 4), c4 = idx % (kTk / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (j0 + c4 * 4 < n)
                v = *reinterpret_cast<const float4 *>(q_in + (int64_t)c * n + j0 + c4 * 4);
            float *d = ql + c * (kTk + 1) + c4 * 4;
            d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
        }
        __syncthreads();
#pragma unroll 4
        for (int jj = 0; jj < kTk; ++jj) {
            const double a = (double)dl[lane_row * (kTk + 1) + jj];
#pragma unroll
            for (int u = 0; u < kAcc; ++u) {
                const int c = wave + 4 * u;
                if (c < r) acc[u] = fma(a, (double)ql[c * (kTk + 1) + jj], acc[u]);
            }
        }
        __syncthreads();
    }
    if (i0 + lane_row < m) {
#pragma unroll
        for (int u = 0; u < kAcc; ++u) {
            const int c = wave + 4 * u;
            if (c < r) out[(int64_t)c * m + i0 + lane_row] = (float)acc[u];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Q_k = delta_k^T * P_hat.  Workgroup: 64 columns of delta over the row range of split
// blockIdx.z; partial results go to slab blockIdx.z (summed afterwards in slab order).
// ---------------------------------------------------------------------------------------------
template <int kAcc>
__global__ __launch_bounds__(kT) void project_q_fma_kernel(PtrPack<const float *> deltas,
                                                           const float *__restrict__ p_hat,
                                                           PtrPack<float *> outs, int64_t m,
                                                           int64_t n, int r, int64_t rows_per_split,
                                                           int64_t slab_stride) {
    extern __shared__ float lds[];
    float *dl = lds;                 // [kTk][kRows]
    float *pl = lds + kTk * kRows;   // [r][kTk + 1]
    const float *__restrict__ delta = deltas.p[blockIdx.y];
    float *__restrict__ out = outs.p[blockIdx.y] + (int64_t)blockIdx.z * slab_stride;
    const int64_t j0 = (int64_t)blockIdx.x * kRows;
    const int lane_col = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t i_begin = (int64_t)blockIdx.z * rows_per_split;
    int64_t i_end = i_begin + rows_per_split;
    if (i_end > m) i_end = m;
    double acc[kAcc];
#pragma unroll
    for (int u = 0; u < kAcc; ++u) acc[u] = 0.0;

    for (int64_t i0 = i_begin; i0 < i_end; i0 += kTk) {
        for (int idx = threadIdx.x; idx < kTk * (kRows / 4); idx += kT) {
            const int ii = idx / (kRows / 4), c4 = idx % (kRows / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + ii < i_end && j0 + c4 * 4 < n)
                v = *reinterpret_cast<const float4 *>(delta + (i0 + ii) * n + j0 + c4 * 4);
            *reinterpret_cast<float4 *>(dl + ii * kRows + c4 * 4) = v;
        }
        for (int idx = threadIdx.x; idx < r * (kTk / 4); idx += kT) {
            const int c = idx / (kTk / 4), c4 = idx % (kTk / 4);
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + c4 * 4 < i_end)  // split ranges are multiples of 4
                v = *reinterpret_cast<const float4 *>(p_hat + (int64_t)c * m + i0 + c4 * 4);
            float *d = pl + c * (kTk + 1) + c4 * 4;
            d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
        }
        __syncthreads();
#pragma unroll 4
        for (int ii = 0; ii < kTk; ++ii) {
            const double a = (double)dl[ii * kRows + lane_col];
#pragma unroll
            for (int u = 0; u < kAcc; ++u) {
                const int c = wave + 4 * u;
                if (c < r) acc[u] = fma(a, (double)pl[c * (kTk + 1) + ii], acc[u]);
            }
        }
        __syncthreads();
    }
    if (j0 + lane_col < n) {
#pragma unroll
        for (int u = 0; u < kAcc; ++u) {
            const int c = wave + 4 * u;
            if (c < r) out[(int64_t)c * n + j0 + lane_col] = (float)acc[u];
        }
    }
}

// out[k][x] = sum_s slabs[k][s][x], s in index order (fixed order: run-to-run identical)
__global__ __launch_bounds__(kT) void sum_slabs_kernel(PtrPack<const float *> slabs,
                                                       PtrPack<float *> outs, int64_t nvec,
                                                       int S, int64_t slab_stride) {
    const int64_t v = (int64_t)blockIdx.x * kT + threadIdx.x;
    if (v >= nvec) return;
    const float *__restrict__ src = slabs.p[blockIdx.y];
    float4 a = reinterpret_cast<const float4 *>(src)[v];
    for (int s = 1; s < S; ++s) {
        const float4 b = reinterpret_cast<const float4 *>(src + (int64_t)s * slab_stride)[v];
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    reinterpret_cast<float4 *>(outs.p[blockIdx.y])[v] = a;
}

int launch_sum_slabs(int K, const PtrPack<const float *> &slabs, const PtrPack<float *> &outs,
                     int64_t count, int S, int64_t slab_stride, hipStream_t st) {
    const int64_t nvec = count >> 2;
    Timed timed(KID_SUM_SLABS, st);
    hipLaunchKernelGGL(sum_slabs_kernel, dim3((unsigned)ceil_div(nvec, kT), (unsigned)K), dim3(kT),
                       0, st, slabs, outs, nvec, S, slab_stride);
    return check_launch("sum_slabs");
}

// ---------------------------------------------------------------------------------------------
// delta_hat = P_hat Q_bar^T on 64 x 64 tiles, 4 x 4 outputs per thread; the epilogue writes the
// tile (optional), subtracts it from the K error buffers (e_k <- delta_k - delta_hat) and, when
// theta is given, applies the Nesterov outer update with the tile as the gradient.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kT) void reconstruct_fma_kernel(const float *__restrict__ p_hat,
                                                             const float *__restrict__ q_bar,
                                                             ReconEpilogue ep, int64_t m,
                                                             int64_t n, int r) {
    __shared__ float pt[kTk][64];
    __shared__ float qt[kTk][64];
    const int64_t i0 = (int64_t)blockIdx.y * 64, j0 = (int64_t)blockIdx.x * 64;
    const int ti = threadIdx.x >> 4, tj = threadIdx.x & 15;
    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0;

    for (int c0 = 0; c0 < r; c0 += kTk) {
        for (int idx = threadIdx.x; idx < kTk * 16; idx += kT) {
            const int cc = idx >> 4, c4 = idx & 15;
            float4 pv = make_float4(0.f, 0.f, 0.f, 0.f), qv = pv;
            if (c0 + cc < r) {
                if (i0 + c4 * 4 < m)
                    pv = *reinterpret_cast<const float4 *>(p_hat + (int64_t)(c0 + cc) * m + i0 + c4 * 4);
                if (j0 + c4 * 4 < n)
                    qv = *reinterpret_cast<const float4 *>(q_bar + (int64_t)(c0 + cc) * n + j0 + c4 * 4);
            }
            *reinterpret_cast<float4 *>(&pt[cc][c4 * 4]) = pv;
            *reinterpret_cast<float4 *>(&qt[cc][c4 * 4]) = qv;
        }
        __syncthreads();
#pragma unroll 4
        for (int cc = 0; cc < kTk; ++cc) {
            const float4 a = *reinterpret_cast<const float4 *>(&pt[cc][ti * 4]);
            const float4 b = *reinterpret_cast<const float4 *>(&qt[cc][tj * 4]);
            const double av[4] = {a.x, a.y, a.z, a.w};
            const double bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) acc[x][y] = fma(av[x], bv[y], acc[x][y]);
        }
        __syncthreads();
    }
    const int64_t j = j0 + tj * 4;
    if (j >= n) return;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int64_t i = i0 + ti * 4 + x;
        if (i >= m) break;
        const float4 d = make_float4((float)acc[x][0], (float)acc[x][1], (float)acc[x][2],
                                     (float)acc[x][3]);
        if (ep.out) *reinterpret_cast<float4 *>(ep.out + i * n + j) = d;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ep.tl_on || ep.apply) t = *reinterpret_cast<const float4 *>(ep.theta + i * n + j);
        for (int k = 0; k < ep.K; ++k) {
            float4 e = *reinterpret_cast<float4 *>(ep.ef.p[k] + i * n + j);
            e.x -= d.x; e.y -= d.y; e.z -= d.z; e.w -= d.w;
            if (ep.tl_on) {
                float4 l;
                if (ep.tl_bf16) {
                    const uint2 b = *reinterpret_cast<const uint2 *>(
                        reinterpret_cast<const uint16_t *>(ep.tl.p[k]) + i * n + j);
                    l = make_float4(__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xFFFF0000u),
                                    __uint_as_float(b.y << 16), __uint_as_float(b.y & 0xFFFF0000u));
                } else {
                    l = *reinterpret_cast<const float4 *>(
                        reinterpret_cast<const float *>(ep.tl.p[k]) + i * n + j);
                }
                e.x = (t.x - l.x) + e.x; e.y = (t.y - l.y) + e.y;
                e.z = (t.z - l.z) + e.z; e.w = (t.w - l.w) + e.w;
            }
            *reinterpret_cast<float4 *>(ep.ef.p[k] + i * n + j) = e;
        }
        if (ep.apply) {
            float4 v = *reinterpret_cast<float4 *>(ep.vel + i * n + j);
            v.x = fmaf(ep.mu, v.x, d.x); v.y = fmaf(ep.mu, v.y, d.y);
            v.z = fmaf(ep.mu, v.z, d.z); v.w = fmaf(ep.mu, v.w, d.w);
            t.x = fmaf(-ep.lr, fmaf(ep.mu, v.x, d.x), t.x);
            t.y = fmaf(-ep.lr, fmaf(ep.mu, v.y, d.y), t.y);
            t.z = fmaf(-ep.lr, fmaf(ep.mu, v.z, d.z), t.z);
            t.w = fmaf(-ep.lr, fmaf(ep.mu, v.w, d.w), t.w);
            *reinterpret_cast<float4 *>(ep.vel + i * n + j) = v;
            *reinterpret_cast<float4 *>(ep.theta + i * n + j) = t;
        }
    }
}

// ---------------------------------------------------------------------------------------------
static int q_splits(int64_t m, int64_t n, int K) {
    const int64_t wgs = ceil_div(n, kRows) * K;
    int64_t s = ceil_div(1024, wgs);
    const int64_t smax = ceil_div(m, 256);
    if (s > smax) s = smax;
    if (s > 64) s = 64;
    return (int)(s < 1 ? 1 : s);
}

size_t fma_project_workspace_bytes(int64_t m, int64_t n, int r, int K) {
    // Q phase: K * S slabs of r x n floats
    return (size_t)K * (size_t)q_splits(m, n, K) * (size_t)r * (size_t)n * sizeof(float);
}

template <typename F>
static int by_rank(int r, F &&f) {
    if (r <= 8) return f(std::integral_constant<int, 2>());
    if (r <= 32) return f(std::integral_constant<int, 8>());
    if (r <= 64) return f(std::integral_constant<int, 16>());
    if (r <= 128) return f(std::integral_constant<int, 32>());
    return f(std::integral_constant<int, 64>());
}

int launch_project_p_fma(int64_t m, int64_t n, int r, int K, const PtrPack<const float *> &delta,
                         const float *q_in, const PtrPack<float *> &out, hipStream_t st) {
    const dim3 grid((unsigned)ceil_div(m, kRows), (unsigned)K);
    const size_t lds = (size_t)(kRows + r) * (kTk + 1) * sizeof(float);
    Timed timed(KID_PROJECT_P, st);
    return by_rank(r, [&](auto acc) {
        hipLaunchKernelGGL((project_p_fma_kernel<decltype(acc)::value>), grid, dim3(kT), lds, st,
                           delta, q_in, out, m, n, r);
        return check_launch("project_p_fma");
    });
}

int launch_project_q_fma(int64_t m, int64_t n, int r, int K, const PtrPack<const float *> &delta,
                         const float *p_hat, const PtrPack<float *> &out, void *workspace,
                         hipStream_t st) {
    const int S = q_splits(m, n, K);
    int64_t rows = ceil_div(m, S);
    rows = ceil_div(rows, kTk) * kTk;
    const int64_t slab = (int64_t)r * n;
    PtrPack<float *> dst = out;
    if (S > 1)
        for (int k = 0; k < K; ++k) dst.p[k] = reinterpret_cast<float *>(workspace) + (int64_t)k * S * slab;
    const dim3 grid((unsigned)ceil_div(n, kRows), (unsigned)K, (unsigned)S);
    const size_t lds = (size_t)(kTk * kRows + r * (kTk + 1)) * sizeof(float);
    int rc;
    {
        Timed timed(KID_PROJECT_Q, st);
        rc = by_rank(r, [&](auto acc) {
        hipLaunchKernelGGL((project_q_fma_kernel<decltype(acc)::value>), grid, dim3(kT), lds, st,
                           delta, p_hat, dst, m, n, r, rows, slab);
        return check_launch("project_q_fma");
        });
    }
    if (rc != DLCX_OK || S == 1) return rc;
    PtrPack<const float *> src;
    for (int k = 0; k < K; ++k) src.p[k] = dst.p[k];
    return launch_sum_slabs(K, src, out, slab, S, slab, st);
}

int launch_reconstruct_fma(int64_t m, int64_t n, int r, const float *p_hat, const float *q_bar,
                           const ReconEpilogue &ep, hipStream_t st) {
    const dim3 grid((unsigned)ceil_div(n, 64), (unsigned)ceil_div(m, 64));
    Timed timed(KID_RECONSTRUCT, st);
    hipLaunchKernelGGL(reconstruct_fma_kernel, grid, dim3(kT), 0, st, p_hat, q_bar, ep, m, n, r);
    return check_launch("reconstruct_fma");
}

}  // namespace dlcx
