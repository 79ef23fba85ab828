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
//
// Every kernel here takes a batch of factors (one descriptor per matrix, passed by value): the
// work per matrix is small and latency-bound, so the matrices of a stage go through each step
// together, one workgroup (or one slice of the grid) per matrix.
#include "common.h"

namespace dlcx {

constexpr int kGramChunk = 512;  // elements of L per partial sum
constexpr int kGT = 256;

int gram_chunks(int64_t L) { return (int)ceil_div(L, kGramChunk); }

// part[chunk][a][b] = sum_{i in chunk} f[a][i] * f[b][i] for the 64 x 64 tile (ta, tb), ta <= tb.
__global__ __launch_bounds__(kGT) void gram_partial_kernel(FactorBatch batch) {
    __shared__ float at[16][64 + 4];
    __shared__ float bt[16][64 + 4];
    const FactorItem it = batch.it[blockIdx.z];
    const float *__restrict__ f = it.f;
    const int64_t L = it.L;
    const int r = it.r;
    const int nt = (r + 63) / 64;
    if ((int)blockIdx.x >= it.nchunks || (int)blockIdx.y >= nt * (nt + 1) / 2) return;
    // tile index -> (ta, tb) with ta <= tb
    int t = blockIdx.y, ta = 0;
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
    double *dst = it.part + (int64_t)blockIdx.x * r * r;
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            const int a = a0 + ty * 4 + x, b = b0 + tx * 4 + y;
            if (a < r && b < r && a <= b) dst[a * r + b] = acc[x][y];
        }
}

// part[0][a][b] <- sum over the chunks, in chunk order, for a <= b: the sum that the one workgroup
// per matrix of the Cholesky and eigenvalue kernels would otherwise form by itself (r^2 x chunks
// loads by one workgroup: 1 - 2 ms of its 3 - 7 ms at r = 256 and L = 28672), here spread over
// the GPU.  Same additions in the same order, so the same bits.
__global__ __launch_bounds__(kGT) void gram_reduce_kernel(FactorBatch batch) {
    const FactorItem it = batch.it[blockIdx.y];
    const int r = it.r;
    const int64_t rr = (int64_t)r * r;
    const int64_t x = (int64_t)blockIdx.x * kGT + threadIdx.x;
    if (x >= rr || it.nchunks < 2) return;
    if (x / r > x % r) return;  // lower triangle: never written, never read
    double s = 0.0;
    for (int c = 0; c < it.nchunks; ++c) s += it.part[(int64_t)c * rr + x];
    it.part[x] = s;
}

// Partial Gram sums of every factor of the batch, then their sum in part[0]: *reduced is the
// batch as the kernels that consume the Gram matrices have to see it (one chunk each).
int launch_gram_partials_batch(const FactorBatch &batch, FactorBatch *reduced, hipStream_t st) {
    int max_chunks = 1, max_tiles = 1, max_r = 1;
    for (int i = 0; i < batch.n; ++i) {
        const int nt = (batch.it[i].r + 63) / 64;
        if (batch.it[i].nchunks > max_chunks) max_chunks = batch.it[i].nchunks;
        if (nt * (nt + 1) / 2 > max_tiles) max_tiles = nt * (nt + 1) / 2;
        if (batch.it[i].r > max_r) max_r = batch.it[i].r;
    }
    const dim3 grid((unsigned)max_chunks, (unsigned)max_tiles, (unsigned)batch.n);
    Timed timed(KID_GRAM, st);
    hipLaunchKernelGGL(gram_partial_kernel, grid, dim3(kGT), 0, st, batch);
    int rc = check_launch("gram_partials");
    if (rc != DLCX_OK) return rc;
    *reduced = batch;
    if (max_chunks < 2) return DLCX_OK;
    const dim3 rgrid((unsigned)ceil_div((int64_t)max_r * max_r, kGT), (unsigned)batch.n);
    hipLaunchKernelGGL(gram_reduce_kernel, rgrid, dim3(kGT), 0, st, batch);
    for (int i = 0; i < batch.n; ++i) reduced->it[i].nchunks = 1;
    return check_launch("gram_reduce");
}

// One workgroup per matrix.  g (r rows of pitch r + 1, fp64, LDS or global) <- sum of the
// partials (upper triangle), scaled to unit diagonal; right-looking Cholesky G = R^T R in place;
// in-place inversion of R column by column; w <- diag(scale) R^-1.  A dead column (pivot <=
// 1e-12, i.e. residual <= 1e-6 of the column norm, or zero norm) gives a zero row of R and a zero
// column of w.
constexpr int kCT = 256;        // threads, small matrices
constexpr int kCTLarge = 1024;  // threads once the matrix no longer fits LDS and lives in L2
constexpr size_t kCholLdsMax = 140 * 1024;

__global__ __launch_bounds__(kCTLarge) void chol_inverse_kernel(FactorBatch batch) {
    extern __shared__ double smem[];
    const FactorItem it = batch.it[blockIdx.x];
    const int r = it.r, nchunks = it.nchunks;
    const int rp = r + 1;                                // odd pitch avoids LDS bank conflicts
    const bool in_lds = (size_t)r * rp * sizeof(double) <= kCholLdsMax;
    double *g = in_lds ? smem : it.g;
    const double *__restrict__ part = it.part;
    double *__restrict__ w = it.w;
    __shared__ double dscale[DLCX_MAX_RANK];             // 1 / column norm (0 for a zero column)
    __shared__ double dinv[DLCX_MAX_RANK];               // 1 / R_cc (0 for a dead column)
    __shared__ double colbuf[DLCX_MAX_RANK];
    __shared__ double psum[(kCTLarge / 256) * 256];      // shares of the inverse's sums
    const int tid = threadIdx.x;
    const int nt = blockDim.x, nty = nt >> 4;            // threads as nty rows of 16
    const int ty = tid >> 4, tx = tid & 15;
    for (int a = ty; a < r; a += nty)
        for (int b = a + tx; b < r; b += 16) {  // sum of the partials in chunk order
            double s = 0.0;
            for (int c = 0; c < nchunks; ++c) s += part[(int64_t)c * r * r + a * r + b];
            g[a * rp + b] = s;
        }
    __syncthreads();
    for (int c = tid; c < r; c += nt) {
        const double d = g[c * rp + c];
        dscale[c] = d > 0.0 ? 1.0 / sqrt(d) : 0.0;
    }
    __syncthreads();
    for (int a = ty; a < r; a += nty)
        for (int b = a + tx; b < r; b += 16) g[a * rp + b] *= dscale[a] * dscale[b];
    __syncthreads();
    for (int c = 0; c < r; ++c) {
        const double piv = g[c * rp + c];
        const bool dead = !(piv > 1e-12);
        const double inv = dead ? 0.0 : 1.0 / sqrt(piv);
        __syncthreads();  // everyone has read the pivot
        if (tid == 0) dinv[c] = inv;
        for (int j = c + tid; j < r; j += nt) g[c * rp + j] *= inv;  // dead: whole row -> 0
        __syncthreads();
        for (int i = c + 1 + ty; i < r; i += nty) {
            const double gi = g[c * rp + i];
            for (int j = c + 1 + tx; j < r; j += 16)
                if (i <= j) g[i * rp + j] -= gi * g[c * rp + j];
        }
        __syncthreads();
    }
    // W = R^-1 in place by back substitution, row by row from the bottom (R W = I: the columns
    // of W are independent, and the rows below row i already hold W).  Row i of R is staged;
    // thread (group, j) adds its share of sum_{l = i+1 .. j} R[i][l] W[l][j], the shares are added
    // in a fixed order, and W[i][j] = -sum / R[i][i] (1 / R[i][i] on the diagonal, 0 for a dead
    // row).  Every access to the matrix in the sum is a row read by consecutive threads.
    const int parts = nt >> 8;  // 1 or 4 groups of 256 threads
    const int jcol = tid & 255, grp = tid >> 8;
    for (int i = r - 1; i >= 0; --i) {
        for (int l = i + 1 + tid; l < r; l += nt) colbuf[l] = g[i * rp + l];
        __syncthreads();
        double s = 0.0;
        if (jcol < r && jcol > i)
            for (int l = i + 1 + grp; l <= jcol; l += parts)
                s = fma(colbuf[l], g[l * rp + jcol], s);
        if (parts > 1) {
            psum[grp * 256 + jcol] = s;
            __syncthreads();
            if (grp == 0) s = ((psum[jcol] + psum[256 + jcol]) + psum[512 + jcol]) + psum[768 + jcol];
        }
        if (grp == 0 && jcol < r && jcol >= i) g[i * rp + jcol] = jcol == i ? dinv[i] : -dinv[i] * s;
        __syncthreads();
    }
    for (int x = tid; x < r * r; x += nt) {
        const int k = x / r, j = x % r;
        w[x] = k <= j ? dscale[k] * g[k * rp + j] : 0.0;
    }
}

// P <- P W in place, fp64 accumulation.  Workgroup: 64 rows of P (= 64 consecutive elements of
// every factor column) staged in LDS; W goes through LDS as well, 16 columns at a time (a
// wavefront's reads of it are broadcasts; straight from memory every one was a round trip to
// L2); thread (row, wave) produces 4 of the 16 columns.  W is upper triangular and stored with
// zeros below the diagonal: column c needs rows k <= c only, and running k up to the last of the
// thread's four columns adds exact zeros to the others.
__global__ __launch_bounds__(kGT) void apply_w_kernel(FactorBatch batch) {
    extern __shared__ float fl[];  // [r][64] floats, then [r][16] doubles of W
    const FactorItem it = batch.it[blockIdx.y];
    float *__restrict__ p = it.f;
    const double *__restrict__ w = it.w;
    const int64_t L = it.L;
    const int r = it.r;
    const int64_t i0 = (int64_t)blockIdx.x * 64;
    if (i0 >= L) return;
    for (int idx = threadIdx.x; idx < r * 16; idx += kGT) {
        const int c = idx >> 4, c4 = idx & 15;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i0 + c4 * 4 < L) v = *reinterpret_cast<const float4 *>(p + (int64_t)c * L + i0 + c4 * 4);
        *reinterpret_cast<float4 *>(fl + c * 64 + c4 * 4) = v;
    }
    __syncthreads();
    const int row = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    double *wl = reinterpret_cast<double *>(fl + (size_t)r * 64);
    for (int c0 = 0; c0 < r; c0 += 16) {
        const int kmax = c0 + 15 < r ? c0 + 15 : r - 1;
        for (int idx = threadIdx.x; idx < (kmax + 1) * 16; idx += kGT) {
            const int k = idx >> 4, ci = idx & 15;
            wl[idx] = c0 + ci < r ? w[k * r + c0 + ci] : 0.0;
        }
        __syncthreads();
        const int cw = c0 + wave * 4;  // this wavefront's four columns
        if (cw < r) {
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            const int kend = cw + 3 < r ? cw + 3 : r - 1;
            // eight k at a time, their LDS reads requested before the first product (one
            // wavefront per SIMD here, nothing else hides the LDS latency: 4.1 -> 2.3 ms for
            // twelve 28672 x 256 factors); the sums keep their order.  (W read through the
            // scalar cache instead of as broadcast LDS reads: 4.9 ms.)
            int k = 0;
            for (; k + 8 <= kend + 1; k += 8) {
                float f[8];
                double wv[8][4];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    f[u] = fl[(k + u) * 64 + row];
#pragma unroll
                    for (int i = 0; i < 4; ++i) wv[u][i] = wl[(k + u) * 16 + wave * 4 + i];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[i] = fma((double)f[u], wv[u][i], acc[i]);
            }
            for (; k <= kend; ++k) {
                const double f = (double)fl[k * 64 + row];
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] = fma(f, wl[k * 16 + wave * 4 + i], acc[i]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (cw + i < r && i0 + row < L) p[(int64_t)(cw + i) * L + i0 + row] = (float)acc[i];
        }
        __syncthreads();  // the tile of W is free again
    }
}

size_t orth_workspace_bytes(int64_t L, int r) {
    // partials + g (pitch r + 1) + w
    return a256x(((size_t)gram_chunks(L) * r * r + (size_t)r * (r + 1) + (size_t)r * r) *
                 sizeof(double));
}

static int cholqr_pass(const FactorBatch &batch, hipStream_t st) {
    FactorBatch summed;  // the same factors with their Gram sums in one chunk
    int rc = launch_gram_partials_batch(batch, &summed, st);
    if (rc != DLCX_OK) return rc;
    size_t g_bytes = 0, a_bytes = 0;
    int64_t max_rows = 1;
    for (int i = 0; i < batch.n; ++i) {
        const size_t r = (size_t)batch.it[i].r;
        const size_t gb = r * (r + 1) * sizeof(double);
        if (gb <= kCholLdsMax && gb > g_bytes) g_bytes = gb;
        const size_t ab = r * 64 * sizeof(float) + r * 16 * sizeof(double);
        if (ab > a_bytes) a_bytes = ab;
        if (ceil_div(batch.it[i].L, 64) > max_rows) max_rows = ceil_div(batch.it[i].L, 64);
    }
    static size_t chol_granted = 0, apply_granted = 0;
    rc = grant_dynamic_lds(reinterpret_cast<const void *>(chol_inverse_kernel), g_bytes, &chol_granted,
                       "chol_inverse attribute");
    if (rc != DLCX_OK) return rc;
    {
        Timed timed(KID_CHOL, st);
        bool large = false;
        for (int i = 0; i < batch.n; ++i)
            large = large || (size_t)batch.it[i].r * (batch.it[i].r + 1) * sizeof(double) > kCholLdsMax;
        hipLaunchKernelGGL(chol_inverse_kernel, dim3((unsigned)batch.n),
                           dim3(large ? kCTLarge : kCT), g_bytes, st, summed);
        rc = check_launch("chol_inverse");
    }
    if (rc != DLCX_OK) return rc;
    rc = grant_dynamic_lds(reinterpret_cast<const void *>(apply_w_kernel), a_bytes, &apply_granted,
                       "apply_w attribute");
    if (rc != DLCX_OK) return rc;
    Timed timed(KID_APPLY_W, st);
    hipLaunchKernelGGL(apply_w_kernel, dim3((unsigned)max_rows, (unsigned)batch.n), dim3(kGT),
                       a_bytes, st, batch);
    return check_launch("apply_w");
}

// Fills the scratch pointers of item i from a workspace of orth_workspace_bytes(L, r) bytes.
void orth_item(FactorItem *it, float *p, int64_t L, int r, void *workspace) {
    it->f = p;
    it->L = L;
    it->r = r;
    it->nchunks = gram_chunks(L);
    it->part = reinterpret_cast<double *>(workspace);
    it->g = it->part + (size_t)it->nchunks * r * r;
    it->w = it->g + (size_t)r * (r + 1);
    it->out = nullptr;
}

int launch_orthonormalize_batch(const FactorBatch &batch, hipStream_t st) {
    if (batch.n == 0) return DLCX_OK;
    int rc = cholqr_pass(batch, st);
    if (rc != DLCX_OK) return rc;
    return cholqr_pass(batch, st);
}

int launch_orthonormalize(int64_t L, int r, float *p_inout, void *workspace, hipStream_t st) {
    FactorBatch b;
    b.n = 1;
    orth_item(&b.it[0], p_inout, L, r, workspace);
    return launch_orthonormalize_batch(b, st);
}

}  // namespace dlcx
