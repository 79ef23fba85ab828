// Orthonormalisation of the averaged factor P_bar (L x r, stored r x L): the thin-QR Q-factor
// with positive diagonal of R, computed as CholeskyQR applied twice with all small-matrix work in
// fp64:
//   1. G = P^T P as fp64 partial sums over chunks of L (fixed chunking, summed in chunk order)
//   2. one workgroup: scale G to unit diagonal, Cholesky G = R^T R, W = R^-1  (r x r, fp64)
//   3. P <- P W, in place, fp64 accumulation
// Scaling the columns of P does not change the Q-factor, and makes the Cholesky factorisation
// insensitive to the very different column norms a warm-started basis produces.  A pivot of the
// scaled matrix is (residual norm / column norm)^2, so the rule "residual <= 1e-6 of the column
// norm => zero column" is a comparison of the pivot with 1e-12.
#include "common.h"

namespace dlcx {

constexpr int kGramChunk = 512;  // elements of L per partial sum
constexpr int kGT = 256;

int gram_chunks(int64_t L) { return (int)ceil_div(L, kGramChunk); }

// part[chunk][a][b] = sum_{i in chunk} f[a][i] * f[b][i] for the 64 x 64 tile (ta, tb), ta <= tb.
__global__ __launch_bounds__(kGT) void gram_partial_kernel(const float *__restrict__ f, int64_t L,
                                                           int r, double *__restrict__ part) {
    __shared__ float at[16][64 + 4];
    __shared__ float bt[16][64 + 4];
    // tile index -> (ta, tb) with ta <= tb
    int t = blockIdx.y, ta = 0, nt = (r + 63) / 64;
    while (t >= nt - ta) {
        t -= nt - ta;
        ++ta;
    }
    const int tb = ta + t;
    const int a0 = ta * 64, b0 = tb * 64;
    const int64_t i_begin = (int64_t)blockIdx.x * kGramChunk;
    int64_t i_end = i_begin + kGramChunk;
    if (i_end > L) i_end = L;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;  // 16 x 16 threads, 4 x 4 each
    double acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[x][y] = 0.0;

    for (int64_t i0 = i_begin; i0 < i_end; i0 += 16) {
        // 64 factor columns x 16 elements for each operand: 256 float4, one per thread
        {
            const int col = threadIdx.x >> 2, c4 = threadIdx.x & 3;
            float4 va = make_float4(0.f, 0.f, 0.f, 0.f), vb = va;
            if (i0 + c4 * 4 < i_end) {
                if (a0 + col < r)
                    va = *reinterpret_cast<const float4 *>(f + (int64_t)(a0 + col) * L + i0 + c4 * 4);
                if (b0 + col < r)
                    vb = *reinterpret_cast<const float4 *>(f + (int64_t)(b0 + col) * L + i0 + c4 * 4);
            }
            at[c4 * 4 + 0][col] = va.x; at[c4 * 4 + 1][col] = va.y;
            at[c4 * 4 + 2][col] = va.z; at[c4 * 4 + 3][col] = va.w;
            bt[c4 * 4 + 0][col] = vb.x; bt[c4 * 4 + 1][col] = vb.y;
            bt[c4 * 4 + 2][col] = vb.z; bt[c4 * 4 + 3][col] = vb.w;
        }
        __syncthreads();
#pragma unroll
        for (int ii = 0; ii < 16; ++ii) {
            const float4 a = *reinterpret_cast<const float4 *>(&at[ii][ty * 4]);
            const float4 b = *reinterpret_cast<const float4 *>(&bt[ii][tx * 4]);
            const double av[4] = {a.x, a.y, a.z, a.w};
            const double bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) acc[x][y] = fma(av[x], bv[y], acc[x][y]);
        }
        __syncthreads();
    }
    double *dst = part + (int64_t)blockIdx.x * r * r;
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            const int a = a0 + ty * 4 + x, b = b0 + tx * 4 + y;
            if (a < r && b < r && a <= b) dst[a * r + b] = acc[x][y];
        }
}

int launch_gram_partials(int64_t L, int r, const float *f, double *partials, hipStream_t st) {
    const int nt = (r + 63) / 64;
    const dim3 grid((unsigned)gram_chunks(L), (unsigned)(nt * (nt + 1) / 2));
    Timed timed(KID_GRAM, st);
    hipLaunchKernelGGL(gram_partial_kernel, grid, dim3(kGT), 0, st, f, L, r, partials);
    return check_launch("gram_partials");
}

// One workgroup.  g (r rows of pitch r + 1, fp64, LDS or global) <- sum of the partials (upper
// triangle), scaled to unit diagonal; right-looking Cholesky G = R^T R in place; in-place
// inversion of R column by column; w <- diag(scale) R^-1.  A dead column (pivot <= 1e-12, i.e.
// residual <= 1e-6 of the column norm, or zero norm) gives a zero row of R and a zero column of w.
constexpr int kCT = 256;

__global__ __launch_bounds__(kCT) void chol_inverse_kernel(const double *__restrict__ part,
                                                           int nchunks, int r,
                                                           double *__restrict__ g_global,
                                                           double *__restrict__ w, int g_in_lds) {
    extern __shared__ double smem[];
    double *g = g_in_lds ? smem : g_global;
    const int rp = r + 1;                                // pitch: odd multiple avoids bank conflicts
    __shared__ double dscale[DLCX_MAX_RANK];             // 1 / column norm (0 for a zero column)
    __shared__ double dinv[DLCX_MAX_RANK];               // 1 / R_cc (0 for a dead column)
    __shared__ double colbuf[DLCX_MAX_RANK];
    const int tid = threadIdx.x;
    const int ty = tid >> 4, tx = tid & 15;
    for (int a = ty; a < r; a += 16)
        for (int b = a + tx; b < r; b += 16) {  // sum of the partials in chunk order
            double s = 0.0;
            for (int c = 0; c < nchunks; ++c) s += part[(int64_t)c * r * r + a * r + b];
            g[a * rp + b] = s;
        }
    __syncthreads();
    for (int c = tid; c < r; c += kCT) {
        const double d = g[c * rp + c];
        dscale[c] = d > 0.0 ? 1.0 / sqrt(d) : 0.0;
    }
    __syncthreads();
    for (int a = ty; a < r; a += 16)
        for (int b = a + tx; b < r; b += 16) g[a * rp + b] *= dscale[a] * dscale[b];
    __syncthreads();
    for (int c = 0; c < r; ++c) {
        const double piv = g[c * rp + c];
        const bool dead = !(piv > 1e-12);
        const double inv = dead ? 0.0 : 1.0 / sqrt(piv);
        __syncthreads();  // everyone has read the pivot
        if (tid == 0) dinv[c] = inv;
        for (int j = c + tid; j < r; j += kCT) g[c * rp + j] *= inv;  // dead: whole row -> 0
        __syncthreads();
        for (int i = c + 1 + ty; i < r; i += 16) {
            const double gi = g[c * rp + i];
            for (int j = c + 1 + tx; j < r; j += 16)
                if (i <= j) g[i * rp + j] -= gi * g[c * rp + j];
        }
        __syncthreads();
    }
    // in-place inverse of the upper triangular R: column j from the inverted leading block
    for (int j = 0; j < r; ++j) {
        for (int l = tid; l < j; l += kCT) colbuf[l] = g[l * rp + j];
        __syncthreads();
        const double dj = dinv[j];
        for (int i = tid; i < j; i += kCT) {
            double s = 0.0;
            for (int l = i; l < j; ++l) s = fma(g[i * rp + l], colbuf[l], s);
            g[i * rp + j] = -dj * s;
        }
        if (tid == 0) g[j * rp + j] = dj;
        __syncthreads();
    }
    for (int x = tid; x < r * r; x += kCT) {
        const int k = x / r, j = x % r;
        w[x] = k <= j ? dscale[k] * g[k * rp + j] : 0.0;
    }
}

// P <- P W in place, fp64 accumulation.  Workgroup: 64 rows of P (= 64 consecutive elements of
// every factor column) staged in LDS; thread (row, wave) produces the columns c = wave, wave+4,..
// W is upper triangular: column c needs rows k <= c only.
__global__ __launch_bounds__(kGT) void apply_w_kernel(float *__restrict__ p, int64_t L, int r,
                                                      const double *__restrict__ w) {
    extern __shared__ float fl[];  // [r][64]
    const int64_t i0 = (int64_t)blockIdx.x * 64;
    for (int idx = threadIdx.x; idx < r * 16; idx += kGT) {
        const int c = idx >> 4, c4 = idx & 15;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i0 + c4 * 4 < L) v = *reinterpret_cast<const float4 *>(p + (int64_t)c * L + i0 + c4 * 4);
        *reinterpret_cast<float4 *>(fl + c * 64 + c4 * 4) = v;
    }
    __syncthreads();
    const int row = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    for (int c = wave; c < r; c += 4) {
        double acc = 0.0;
        for (int k = 0; k <= c; ++k) acc = fma((double)fl[k * 64 + row], w[k * r + c], acc);
        if (i0 + row < L) p[(int64_t)c * L + i0 + row] = (float)acc;
    }
}

size_t orth_workspace_bytes(int64_t L, int r) {
    // partials + g (pitch r + 1) + w
    return ((size_t)gram_chunks(L) * r * r + (size_t)r * (r + 1) + (size_t)r * r) * sizeof(double);
}

static int cholqr_pass(int64_t L, int r, float *p, double *part, double *g, double *w,
                       hipStream_t st) {
    int rc = launch_gram_partials(L, r, p, part, st);
    if (rc != DLCX_OK) return rc;
    const size_t g_bytes = (size_t)r * (r + 1) * sizeof(double);
    const int in_lds = g_bytes <= 140 * 1024 ? 1 : 0;
    if (in_lds && g_bytes > 48 * 1024) {
        rc = note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(chol_inverse_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)g_bytes),
                      "chol_inverse attribute");
        if (rc != DLCX_OK) return rc;
    }
    {
        Timed timed(KID_CHOL, st);
        hipLaunchKernelGGL(chol_inverse_kernel, dim3(1), dim3(kCT), in_lds ? g_bytes : 0, st, part,
                           gram_chunks(L), r, g, w, in_lds);
        rc = check_launch("chol_inverse");
    }
    if (rc != DLCX_OK) return rc;
    const size_t lds = (size_t)r * 64 * sizeof(float);
    if (lds > 48 * 1024) {
        rc = note_hip(hipFuncSetAttribute(reinterpret_cast<const void *>(apply_w_kernel),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds),
                      "apply_w attribute");
        if (rc != DLCX_OK) return rc;
    }
    Timed timed(KID_APPLY_W, st);
    hipLaunchKernelGGL(apply_w_kernel, dim3((unsigned)ceil_div(L, 64)), dim3(kGT), lds, st, p, L, r,
                       w);
    return check_launch("apply_w");
}

int launch_orthonormalize(int64_t L, int r, float *p_inout, void *workspace, hipStream_t st) {
    double *part = reinterpret_cast<double *>(workspace);
    double *g = part + (size_t)gram_chunks(L) * r * r;
    double *w = g + (size_t)r * (r + 1);
    int rc = cholqr_pass(L, r, p_inout, part, g, w, st);
    if (rc != DLCX_OK) return rc;
    return cholqr_pass(L, r, p_inout, part, g, w, st);
}

}  // namespace dlcx
