// Shared host/device declarations of the dlcx HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/dlcx.h"

namespace dlcx {

// K device pointers passed to a kernel by value.
template <typename T>
struct PtrPack {
    T p[DLCX_MAX_WORKERS];
};

// Records a HIP error for dlcx_last_hip_error(); returns DLCX_ELAUNCH or DLCX_OK.
int note_hip(hipError_t e, const char *where);

inline int check_launch(const char *where) { return note_hip(hipGetLastError(), where); }

// Raises `kernel`'s limit of dynamic LDS to at least `bytes` (needed above 48 KB).  *granted
// remembers the largest value set so far for that kernel; check, call and update happen under
// one process-wide lock, so two host threads that launch on two streams can neither skip a
// needed call nor leave a smaller limit behind a larger request.
int grant_dynamic_lds(const void *kernel, size_t bytes, size_t *granted, const char *what);

// Optional per-kernel timing (dlcx_profile_*): when enabled, a Timed object brackets one kernel
// launch with two HIP events on the launch stream.  Off by default; costs nothing when off.
enum KernelId {
    KID_DELTA_EF = 0, KID_NESTEROV, KID_QUANTIZE, KID_DEQUANT_AVG, KID_PACK, KID_PROJECT_P,
    KID_PROJECT_Q, KID_SUM_SLABS, KID_RECONSTRUCT, KID_GRAM, KID_CHOL, KID_APPLY_W, KID_JACOBI,
    KID_ROUND, KID_QUANT_ROUND, KID_REQUANT, KID_EF_UPDATE,
    KID_MFMA_PEAK, KID_TRAFFIC_PROBE, KID_COUNT
};
struct Timed {
    Timed(int kid, hipStream_t st);
    ~Timed();
    int slot;
    hipStream_t st;
    void *stop;  // the closing event of this launch's record
};

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// ---- streaming kernels (k_stream.hip) -------------------------------------------------
int launch_delta_ef(const float *theta_g, const void *theta_l, int dtype, float *ef,
                    int64_t numel, hipStream_t st);
int launch_nesterov(float *theta, float *v, const float *g, int64_t numel, float lr, float mu,
                    hipStream_t st);

// ---- quantiser (k_quant.hip) ----------------------------------------------------------
// K factors of `count` floats each; x.p[k] -> codes.p[k], scales.p[k].
int launch_quantize(int K, const PtrPack<const float *> &x, int64_t count, int qbits, int group,
                    const PtrPack<uint8_t *> &codes, const PtrPack<float *> &scales,
                    hipStream_t st);
int launch_dequant_average(int K, const PtrPack<const uint8_t *> &codes,
                           const PtrPack<const float *> &scales, int64_t count, int qbits,
                           int group, float *mean_out, hipStream_t st);

// ---- quantise-only outer step (k_qround.hip) ------------------------------------------
int launch_quant_round(int64_t numel, int qbits, int group, int K, const PtrPack<const void *> &tl,
                       int tl_dtype, const PtrPack<float *> &ef, float *theta, float *vel, double lr,
                       double mu, bool has_prev, const PtrPack<const uint8_t *> &pcodes,
                       const PtrPack<const float *> &pscales, bool requant,
                       const PtrPack<uint8_t *> &codes, const PtrPack<float *> &scales,
                       hipStream_t st);
int launch_requantize(float *x, int64_t count, int qbits, int group, hipStream_t st);
int launch_ef_update(int K, const PtrPack<float *> &ef, const float *d, int64_t numel,
                     hipStream_t st);

// ---- measurement aid (k_peak.hip) -------------------------------------------------------
int launch_mfma_peak(int workgroups, int iters, int operands, float *out, hipStream_t st);
int launch_traffic_probe(int K, const PtrPack<float *> &ef, const PtrPack<const void *> &tl,
                         bool tl_bf16, float *theta, float *vel, int64_t numel, hipStream_t st);

// ---- rank-r products ------------------------------------------------------------------
// P_k = delta_k * Q_in   (delta m x n, q_in r x n, out r x m)
int launch_project_p(int mma, int64_t m, int64_t n, int r, int K,
                     const PtrPack<const float *> &delta, const float *q_in,
                     const PtrPack<float *> &out, void *workspace, hipStream_t st);
// Q_k = delta_k^T * P_hat (p_hat r x m, out r x n)
int launch_project_q(int mma, int64_t m, int64_t n, int r, int K,
                     const PtrPack<const float *> &delta, const float *p_hat,
                     const PtrPack<float *> &out, void *workspace, hipStream_t st);
// What happens to each tile d of delta_hat = P_hat Q_bar^T, in this order:
//   out            : d is written
//   K > 0          : e_k <- e_k - d                     (error buffers of Alg. 2)
//   tl_on          : e_k <- (theta - theta_l,k) + e_k   (next pseudo-gradient, same buffer)
//   apply          : vel <- mu vel + d ; theta <- theta - lr (d + mu vel)   (OuterOpt)
struct ReconEpilogue {
    float *out;
    int K;
    PtrPack<float *> ef;
    PtrPack<const void *> tl;
    int tl_on, tl_bf16;
    float *theta, *vel;
    int apply;
    float lr, mu;
};
int launch_reconstruct(int mma, int64_t m, int64_t n, int r, const float *p_hat,
                       const float *q_bar, const ReconEpilogue &ep, void *workspace,
                       hipStream_t st);
size_t project_workspace_bytes(int mma, int64_t m, int64_t n, int r, int K);
size_t reconstruct_workspace_bytes(int mma, int64_t m, int64_t n, int r);

// ---- orthonormalisation and effective rank (k_orth.hip, k_rank.hip) ---------------------
inline size_t a256x(size_t x) { return (x + 255) & ~(size_t)255; }
// One r x L factor and its fp64 scratch; a batch of them is passed to a kernel by value.
constexpr int kMaxBatch = 64;
struct FactorItem {
    float *f;        // the factor (read by the Gram kernel, rewritten by apply_w)
    int64_t L;
    int32_t r, nchunks;
    double *part;    // nchunks x r x r partial Gram sums (upper triangles)
    double *g;       // r x (r + 1): Cholesky scratch, or the Jacobi matrix
    double *w;       // r x r: inverse factor (orthonormalisation only)
    int32_t *out;    // r' (effective rank only)
};
struct FactorBatch {
    int n;
    FactorItem it[kMaxBatch];
};
size_t orth_workspace_bytes(int64_t L, int r);
void orth_item(FactorItem *it, float *p, int64_t L, int r, void *workspace);
int launch_orthonormalize(int64_t L, int r, float *p_inout, void *workspace, hipStream_t st);
int launch_orthonormalize_batch(const FactorBatch &batch, hipStream_t st);
size_t effrank_workspace_bytes(int64_t L, int r);
void effrank_item(FactorItem *it, const float *q_bar, int64_t L, int r, int32_t *out,
                  void *workspace);
int launch_effective_rank(int64_t L, int r, const float *q_bar, double tau, int32_t *rprime_dev,
                          void *workspace, hipStream_t st);
int launch_effective_rank_batch(const FactorBatch &batch, double tau, hipStream_t st);
// fp64 Gram matrix partials of r x L factors: part[chunk][a][b] for a <= b (others untouched)
int gram_chunks(int64_t L);
int launch_gram_partials_batch(const FactorBatch &batch, FactorBatch *reduced, hipStream_t st);

}  // namespace dlcx
