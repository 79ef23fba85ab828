// Entry points of libdlcx_hip.so: argument validation on the host, then kernel launches.
// Nothing here allocates or synchronises, except dlcx_select_rank which returns integers.
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "common.h"

namespace dlcx {

static thread_local std::string g_last_error;

int note_hip(hipError_t e, const char *where) {
    if (e == hipSuccess) return DLCX_OK;
    g_last_error = std::string(where) + ": " + hipGetErrorString(e);
    return DLCX_ELAUNCH;
}

int grant_dynamic_lds(const void *kernel, size_t bytes, size_t *granted, const char *what) {
    if (bytes <= 48 * 1024) return DLCX_OK;
    static std::mutex mu;
    std::lock_guard<std::mutex> lock(mu);
    if (bytes <= *granted) return DLCX_OK;
    int rc = note_hip(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                          (int)bytes), what);
    if (rc == DLCX_OK) *granted = bytes;
    return rc;
}

// ---- optional per-kernel timing ---------------------------------------------------------
struct ProfRec {
    int kid;
    hipEvent_t a, b;
};
static std::mutex g_prof_mutex;  // guards g_prof_on and g_prof (launches may come from several threads)
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof;

Timed::Timed(int kid, hipStream_t s) : slot(-1), st(s), stop(nullptr) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof_on) return;
    ProfRec r;
    r.kid = kid;
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) {
        (void)hipEventDestroy(r.a);
        return;
    }
    if (hipEventRecord(r.a, st) != hipSuccess) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
        return;
    }
    g_prof.push_back(r);
    slot = (int)g_prof.size() - 1;
    stop = r.b;  // the record may move when another thread appends: keep the handle itself
}
Timed::~Timed() {
    if (slot >= 0) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(stop), st);
}

// k_gemm_fma.hip
int launch_project_p_fma(int64_t, int64_t, int, int, const PtrPack<const float *> &, const float *,
                         const PtrPack<float *> &, hipStream_t);
int launch_project_q_fma(int64_t, int64_t, int, int, const PtrPack<const float *> &, const float *,
                         const PtrPack<float *> &, void *, hipStream_t);
int launch_reconstruct_fma(int64_t, int64_t, int, const float *, const float *,
                           const ReconEpilogue &, hipStream_t);
size_t fma_project_workspace_bytes(int64_t, int64_t, int, int);
// k_gemm_mfma.hip
int launch_project_p_mfma(int, int64_t, int64_t, int, int, const PtrPack<const float *> &,
                          const float *, const PtrPack<float *> &, void *, hipStream_t);
int launch_project_q_mfma(int, int64_t, int64_t, int, int, const PtrPack<const float *> &,
                          const float *, const PtrPack<float *> &, void *, hipStream_t);
int launch_reconstruct_mfma(int, int64_t, int64_t, int, const float *, const float *,
                            const ReconEpilogue &, void *, hipStream_t);
size_t mfma_project_workspace_bytes(int, int64_t, int64_t, int, int);
size_t mfma_reconstruct_workspace_bytes(int, int64_t, int64_t, int);
size_t mfma_round_workspace_bytes(int, int64_t, int64_t, int, int, int);
int launch_round_mfma(int, int64_t, int64_t, int, int, const float *, const float *, const float *,
                      const ReconEpilogue &, const PtrPack<float *> &, void *, hipStream_t);

static bool group_ok(int g) { return g == 16 || g == 32 || g == 64 || g == 128 || g == 256; }

static int check_desc(const dlcx_desc *d) {
    if (!d) return DLCX_EINVAL;
    if (d->m <= 0 || d->n <= 0) return DLCX_EINVAL;
    if (d->qbits != 4 && d->qbits != 8) return DLCX_EINVAL;
    if (!group_ok(d->group)) return DLCX_EINVAL;
    if (d->m % d->group || d->n % d->group) return DLCX_EINVAL;
    if (d->r < 1 || d->r > DLCX_MAX_RANK || d->r > d->m || d->r > d->n) return DLCX_EINVAL;
    if (d->mma < DLCX_MMA_FMA || d->mma > DLCX_MMA_F16) return DLCX_EINVAL;
    return DLCX_OK;
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static size_t factor_region_bytes(const dlcx_desc *d, int K) {
    const int64_t lmax = d->m > d->n ? d->m : d->n;
    return align256((size_t)K * d->r * lmax * sizeof(float));
}

size_t project_workspace_bytes(int mma, int64_t m, int64_t n, int r, int K) {
    if (mma == DLCX_MMA_FMA) return fma_project_workspace_bytes(m, n, r, K);
    return mfma_project_workspace_bytes(mma, m, n, r, K);
}

int launch_project_p(int mma, int64_t m, int64_t n, int r, int K,
                     const PtrPack<const float *> &delta, const float *q_in,
                     const PtrPack<float *> &out, void *workspace, hipStream_t st) {
    if (mma == DLCX_MMA_FMA) return launch_project_p_fma(m, n, r, K, delta, q_in, out, st);
    return launch_project_p_mfma(mma, m, n, r, K, delta, q_in, out, workspace, st);
}

int launch_project_q(int mma, int64_t m, int64_t n, int r, int K,
                     const PtrPack<const float *> &delta, const float *p_hat,
                     const PtrPack<float *> &out, void *workspace, hipStream_t st) {
    if (mma == DLCX_MMA_FMA) return launch_project_q_fma(m, n, r, K, delta, p_hat, out, workspace, st);
    return launch_project_q_mfma(mma, m, n, r, K, delta, p_hat, out, workspace, st);
}

size_t reconstruct_workspace_bytes(int mma, int64_t m, int64_t n, int r) {
    if (mma == DLCX_MMA_FMA) return 0;
    return mfma_reconstruct_workspace_bytes(mma, m, n, r);
}

int launch_reconstruct(int mma, int64_t m, int64_t n, int r, const float *p_hat,
                       const float *q_bar, const ReconEpilogue &ep, void *workspace,
                       hipStream_t st) {
    if (mma == DLCX_MMA_FMA) return launch_reconstruct_fma(m, n, r, p_hat, q_bar, ep, st);
    return launch_reconstruct_mfma(mma, m, n, r, p_hat, q_bar, ep, workspace, st);
}

}  // namespace dlcx

using namespace dlcx;

extern "C" {

const char *dlcx_strerror(int code) {
    switch (code) {
        case DLCX_OK: return "ok";
        case DLCX_EINVAL: return "invalid argument";
        case DLCX_EUNSUPPORTED: return "unsupported configuration";
        case DLCX_ELAUNCH: return "HIP runtime error";
        case DLCX_ETOOBIG: return "larger than the fixed scratch of this entry point";
        default: return "unknown error code";
    }
}

const char *dlcx_last_hip_error(void) { return g_last_error.c_str(); }

static const char *const kKernelNames[KID_COUNT] = {
    "delta_ef", "outer_nesterov", "quantize", "dequant_average", "pack_fragments", "project_p",
    "project_q", "sum_slabs", "reconstruct", "gram_partials", "chol_inverse", "apply_w",
    "jacobi_rank", "round_fused", "quant_round", "requantize", "ef_update",
    "mfma_peak", "traffic_probe"};

int dlcx_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    for (auto &r : g_prof) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_prof.clear();
    g_prof_on = on != 0;
    return DLCX_OK;
}

int dlcx_profile_kernels(void) { return KID_COUNT; }

const char *dlcx_profile_name(int kernel_id) {
    return kernel_id >= 0 && kernel_id < KID_COUNT ? kKernelNames[kernel_id] : "";
}

int dlcx_profile_read(int kernel_id, double *total_ms_host, int64_t *launches_host) {
    if (kernel_id < 0 || kernel_id >= KID_COUNT || !total_ms_host || !launches_host)
        return DLCX_EINVAL;
    double total = 0.0;
    int64_t count = 0;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    for (auto &r : g_prof) {
        if (r.kid != kernel_id) continue;
        int rc = note_hip(hipEventSynchronize(r.b), "profile sync");
        if (rc != DLCX_OK) return rc;
        float ms = 0.f;
        rc = note_hip(hipEventElapsedTime(&ms, r.a, r.b), "profile elapsed");
        if (rc != DLCX_OK) return rc;
        total += ms;
        ++count;
    }
    *total_ms_host = total;
    *launches_host = count;
    return DLCX_OK;
}

size_t dlcx_payload_bytes(const dlcx_desc *desc, int phase, size_t *codes_bytes,
                          size_t *scales_bytes) {
    if (check_desc(desc) != DLCX_OK || (phase != DLCX_PHASE_P && phase != DLCX_PHASE_Q)) return 0;
    const size_t count = (size_t)desc->r * (size_t)(phase == DLCX_PHASE_P ? desc->m : desc->n);
    const size_t cb = desc->qbits == 4 ? count / 2 : count;
    const size_t sb = count / desc->group * sizeof(float);
    if (codes_bytes) *codes_bytes = cb;
    if (scales_bytes) *scales_bytes = sb;
    return cb + sb;
}

size_t dlcx_workspace_bytes(const dlcx_desc *desc, int K) {
    if (check_desc(desc) != DLCX_OK || K < 1 || K > DLCX_MAX_WORKERS) return 0;
    const int64_t lmax = desc->m > desc->n ? desc->m : desc->n;
    const size_t proj = factor_region_bytes(desc, K) +
                        project_workspace_bytes(desc->mma, desc->m, desc->n, desc->r, K);
    const size_t orth = orth_workspace_bytes(lmax, desc->r);
    const size_t rank = effrank_workspace_bytes(lmax, desc->r);
    size_t rec = reconstruct_workspace_bytes(desc->mma, desc->m, desc->n, desc->r);
    if (desc->mma != DLCX_MMA_FMA) {
        const size_t rnd = factor_region_bytes(desc, K) +
                           mfma_round_workspace_bytes(desc->mma, desc->m, desc->n, desc->r, desc->r, K);
        if (rnd > rec) rec = rnd;
    }
    size_t w = proj > orth ? proj : orth;
    if (rank > w) w = rank;
    if (rec > w) w = rec;
    return align256(w);
}

size_t dlcx_select_rank_workspace_bytes(const dlcx_desc *descs, int n_matrices) {
    if (n_matrices < 0 || (n_matrices > 0 && !descs)) return 0;
    size_t total = align256((size_t)(n_matrices > 0 ? n_matrices : 1) * sizeof(int32_t));
    for (int i = 0; i < n_matrices; ++i) {
        if (check_desc(&descs[i]) != DLCX_OK) return 0;
        total += effrank_workspace_bytes(descs[i].n, descs[i].r);
    }
    return total;
}

int dlcx_delta_ef(const float *theta_g, const void *theta_l, int theta_l_dtype, float *ef_inout,
                  int64_t numel, void *stream) {
    if (numel < 0) return DLCX_EINVAL;
    if (theta_l_dtype != DLCX_F32 && theta_l_dtype != DLCX_BF16) return DLCX_EINVAL;
    if (numel == 0) return DLCX_OK;
    if (!theta_g || !theta_l || !ef_inout) return DLCX_EINVAL;
    if (!aligned16(theta_g) || !aligned16(theta_l) || !aligned16(ef_inout)) return DLCX_EINVAL;
    return launch_delta_ef(theta_g, theta_l, theta_l_dtype, ef_inout, numel, as_stream(stream));
}

int dlcx_outer_nesterov(float *theta_g, float *v, const float *delta_hat, int64_t numel, float lr,
                        float mu, void *stream) {
    if (numel < 0) return DLCX_EINVAL;
    if (numel == 0) return DLCX_OK;
    if (!theta_g || !v || !delta_hat) return DLCX_EINVAL;
    if (!aligned16(theta_g) || !aligned16(v) || !aligned16(delta_hat)) return DLCX_EINVAL;
    if (!(lr == lr) || !(mu == mu)) return DLCX_EINVAL;
    return launch_nesterov(theta_g, v, delta_hat, numel, lr, mu, as_stream(stream));
}

int dlcx_quant_round(int64_t numel, int qbits, int group, int K,
                     const void *const *theta_l_host, int theta_l_dtype,
                     float *const *ef_inout_host, float *theta_g, float *v, double lr, double mu,
                     const uint8_t *const *prev_codes_host, const float *const *prev_scales_host,
                     int requant, uint8_t *const *codes_out_host, float *const *scales_out_host,
                     void *stream) {
    if (numel < 0 || (qbits != 4 && qbits != 8) || !group_ok(group) || numel % group)
        return DLCX_EINVAL;
    if (K < 1 || K > DLCX_MAX_WORKERS) return DLCX_EINVAL;
    if (theta_l_dtype != DLCX_F32 && theta_l_dtype != DLCX_BF16) return DLCX_EINVAL;
    if ((prev_codes_host == nullptr) != (prev_scales_host == nullptr)) return DLCX_EINVAL;
    if (numel == 0) return DLCX_OK;
    if (!theta_l_host || !ef_inout_host || !theta_g || !codes_out_host || !scales_out_host)
        return DLCX_EINVAL;
    const bool has_prev = prev_codes_host != nullptr;
    if (has_prev && !v) return DLCX_EINVAL;
    if (!aligned16(theta_g) || (v && !aligned16(v))) return DLCX_EINVAL;
    if (!(lr == lr) || !(mu == mu)) return DLCX_EINVAL;
    PtrPack<const void *> tl;
    PtrPack<float *> ef;
    PtrPack<const uint8_t *> pc;
    PtrPack<const float *> ps;
    PtrPack<uint8_t *> cs;
    PtrPack<float *> ss;
    for (int k = 0; k < K; ++k) {
        if (!theta_l_host[k] || !ef_inout_host[k] || !codes_out_host[k] || !scales_out_host[k])
            return DLCX_EINVAL;
        if (!aligned16(theta_l_host[k]) || !aligned16(ef_inout_host[k]) ||
            !aligned16(codes_out_host[k]) || !aligned16(scales_out_host[k]))
            return DLCX_EINVAL;
        tl.p[k] = theta_l_host[k];
        ef.p[k] = ef_inout_host[k];
        cs.p[k] = codes_out_host[k];
        ss.p[k] = scales_out_host[k];
        pc.p[k] = nullptr;
        ps.p[k] = nullptr;
        if (has_prev) {
            if (!prev_codes_host[k] || !prev_scales_host[k]) return DLCX_EINVAL;
            if (!aligned16(prev_codes_host[k]) || !aligned16(prev_scales_host[k]))
                return DLCX_EINVAL;
            pc.p[k] = prev_codes_host[k];
            ps.p[k] = prev_scales_host[k];
        }
    }
    return launch_quant_round(numel, qbits, group, K, tl, theta_l_dtype, ef, theta_g, v, lr, mu,
                              has_prev, pc, ps, requant != 0, cs, ss, as_stream(stream));
}

int dlcx_mfma_peak_probe(int workgroups, int iters, int operands, float *out, void *stream) {
    if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 24)) return DLCX_EINVAL;
    if ((operands != 0 && operands != 1) || !out || !aligned16(out)) return DLCX_EINVAL;
    return launch_mfma_peak(workgroups, iters, operands, out, as_stream(stream));
}

int dlcx_traffic_probe(int K, const void *const *theta_l_host, int theta_l_dtype,
                       float *const *ef_inout_host, float *theta_g, float *v, int64_t numel,
                       void *stream) {
    if (K < 1 || K > DLCX_MAX_WORKERS || numel < 0 || numel % 1024) return DLCX_EINVAL;
    if (theta_l_dtype != DLCX_F32 && theta_l_dtype != DLCX_BF16) return DLCX_EINVAL;
    if (numel / 1024 > 0x7fffffff) return DLCX_EINVAL;
    if (numel == 0) return DLCX_OK;
    if (!theta_l_host || !ef_inout_host || !theta_g || !v || !aligned16(theta_g) || !aligned16(v))
        return DLCX_EINVAL;
    PtrPack<float *> ef;
    PtrPack<const void *> tl;
    for (int k = 0; k < K; ++k) {
        if (!theta_l_host[k] || !ef_inout_host[k] || !aligned16(theta_l_host[k]) ||
            !aligned16(ef_inout_host[k]))
            return DLCX_EINVAL;
        ef.p[k] = ef_inout_host[k];
        tl.p[k] = theta_l_host[k];
    }
    return launch_traffic_probe(K, ef, tl, theta_l_dtype == DLCX_BF16, theta_g, v, numel,
                                as_stream(stream));
}

int dlcx_ef_update(int K, float *const *ef_inout_host, const float *delta_hat, int64_t numel,
                   void *stream) {
    if (K < 0 || K > DLCX_MAX_WORKERS || numel < 0) return DLCX_EINVAL;
    if (K == 0 || numel == 0) return DLCX_OK;
    if (!ef_inout_host || !delta_hat || !aligned16(delta_hat)) return DLCX_EINVAL;
    PtrPack<float *> ef;
    for (int k = 0; k < K; ++k) {
        if (!ef_inout_host[k] || !aligned16(ef_inout_host[k])) return DLCX_EINVAL;
        ef.p[k] = ef_inout_host[k];
    }
    return launch_ef_update(K, ef, delta_hat, numel, as_stream(stream));
}

int dlcx_requantize(float *x_inout, int64_t count, int qbits, int group, void *stream) {
    if (count < 0 || (qbits != 4 && qbits != 8) || !group_ok(group) || count % group)
        return DLCX_EINVAL;
    if (count == 0) return DLCX_OK;
    if (!x_inout || !aligned16(x_inout)) return DLCX_EINVAL;
    return launch_requantize(x_inout, count, qbits, group, as_stream(stream));
}

double dlcx_comm_seconds(double payload_bytes, int clusters, double bits_per_second) {
    if (!(payload_bytes >= 0.0) || clusters < 1 || !(bits_per_second > 0.0)) return -1.0;
    const double between = 2.0 * (double)(clusters - 1) / (double)clusters * payload_bytes;
    return between * 8.0 / bits_per_second;
}

static double stage_payload_bytes(const dlcx_desc *descs, int n, int32_t r, double extra,
                                  int iters) {
    double factors = 0.0;
    for (int a = 0; a < n; ++a) {
        dlcx_desc d = descs[a];
        const int64_t side = d.m < d.n ? d.m : d.n;
        d.r = r < side ? r : (int32_t)side;
        factors += (double)dlcx_payload_bytes(&d, DLCX_PHASE_P, nullptr, nullptr);
        factors += (double)dlcx_payload_bytes(&d, DLCX_PHASE_Q, nullptr, nullptr);
    }
    return extra + (double)iters * factors;
}

int dlcx_plan_overlap(const dlcx_desc *descs_host, int n_matrices, double extra_bytes,
                      int power_iters, int32_t rmin, int32_t rmax, int clusters,
                      double bits_per_second, double step_seconds, int32_t H, int32_t *r_out,
                      int32_t *H_out, double *comm_seconds_out) {
    if (n_matrices < 0 || (n_matrices > 0 && !descs_host) || !(extra_bytes >= 0.0)) return DLCX_EINVAL;
    if (power_iters < 1 || power_iters > 1024) return DLCX_EINVAL;
    if (rmin < 1 || rmax < rmin || rmax > DLCX_MAX_RANK || clusters < 1 || H < 1) return DLCX_EINVAL;
    if (!(bits_per_second > 0.0) || !(step_seconds > 0.0)) return DLCX_EINVAL;
    if (!r_out || !H_out || !comm_seconds_out) return DLCX_EINVAL;
    for (int a = 0; a < n_matrices; ++a) {
        dlcx_desc d = descs_host[a];
        d.r = 1;  // the rank field of the inputs is not used
        if (check_desc(&d) != DLCX_OK) return DLCX_EINVAL;
    }
    const double budget = (double)H * step_seconds;
    int32_t best = 0;
    for (int32_t r = rmin; r <= rmax; ++r) {  // the payload grows with r: keep the last that fits
        const double t = dlcx_comm_seconds(
            stage_payload_bytes(descs_host, n_matrices, r, extra_bytes, power_iters), clusters,
            bits_per_second);
        if (t <= budget) best = r;
        else break;
    }
    if (best >= rmin) {
        *r_out = best;
        *H_out = H;
        *comm_seconds_out = dlcx_comm_seconds(
            stage_payload_bytes(descs_host, n_matrices, best, extra_bytes, power_iters), clusters,
            bits_per_second);
        return DLCX_OK;
    }
    const double t = dlcx_comm_seconds(
        stage_payload_bytes(descs_host, n_matrices, rmin, extra_bytes, power_iters), clusters,
        bits_per_second);
    double h = t / step_seconds;
    int64_t hi = (int64_t)h;
    if ((double)hi < h) ++hi;
    if (hi < 1) hi = 1;
    if (hi > INT32_MAX) return DLCX_EINVAL;
    *r_out = rmin;
    *H_out = (int32_t)hi;
    *comm_seconds_out = t;
    return DLCX_OK;
}

int dlcx_project(const dlcx_desc *desc, int phase, int K, const float *const *deltas_host,
                 const float *basis, float *const *factors_out_host, void *workspace,
                 void *stream) {
    int rc = check_desc(desc);
    if (rc != DLCX_OK) return rc;
    if (phase != DLCX_PHASE_P && phase != DLCX_PHASE_Q) return DLCX_EINVAL;
    if (K < 1 || K > DLCX_MAX_WORKERS || !deltas_host || !factors_out_host || !basis)
        return DLCX_EINVAL;
    if (!aligned16(basis) || !aligned16(workspace)) return DLCX_EINVAL;
    PtrPack<const float *> d;
    PtrPack<float *> o;
    for (int k = 0; k < K; ++k) {
        if (!deltas_host[k] || !factors_out_host[k]) return DLCX_EINVAL;
        if (!aligned16(deltas_host[k]) || !aligned16(factors_out_host[k])) return DLCX_EINVAL;
        d.p[k] = deltas_host[k];
        o.p[k] = factors_out_host[k];
    }
    if (project_workspace_bytes(desc->mma, desc->m, desc->n, desc->r, K) > 0 && !workspace)
        return DLCX_EINVAL;
    if (phase == DLCX_PHASE_P)
        return launch_project_p(desc->mma, desc->m, desc->n, desc->r, K, d, basis, o, workspace,
                                as_stream(stream));
    return launch_project_q(desc->mma, desc->m, desc->n, desc->r, K, d, basis, o, workspace,
                            as_stream(stream));
}

int dlcx_quantize(const float *x, int64_t count, int qbits, int group, uint8_t *codes_out,
                  float *scales_out, void *stream) {
    if (count < 0 || (qbits != 4 && qbits != 8) || !group_ok(group) || count % group)
        return DLCX_EINVAL;
    if (count == 0) return DLCX_OK;
    if (!x || !codes_out || !scales_out) return DLCX_EINVAL;
    if (!aligned16(x) || !aligned16(codes_out) || !aligned16(scales_out)) return DLCX_EINVAL;
    PtrPack<const float *> xs;
    PtrPack<uint8_t *> cs;
    PtrPack<float *> ss;
    xs.p[0] = x;
    cs.p[0] = codes_out;
    ss.p[0] = scales_out;
    return launch_quantize(1, xs, count, qbits, group, cs, ss, as_stream(stream));
}

int dlcx_compress_batched(const dlcx_desc *desc, int phase, int K,
                          const float *const *deltas_host, const float *basis,
                          uint8_t *const *codes_out_host, float *const *scales_out_host,
                          void *workspace, void *stream) {
    int rc = check_desc(desc);
    if (rc != DLCX_OK) return rc;
    if (phase != DLCX_PHASE_P && phase != DLCX_PHASE_Q) return DLCX_EINVAL;
    if (K < 1 || K > DLCX_MAX_WORKERS || !deltas_host || !codes_out_host || !scales_out_host ||
        !basis || !workspace)
        return DLCX_EINVAL;
    if (!aligned16(workspace)) return DLCX_EINVAL;
    const int64_t L = phase == DLCX_PHASE_P ? desc->m : desc->n;
    const int64_t count = (int64_t)desc->r * L;
    float *factors[DLCX_MAX_WORKERS];
    PtrPack<const float *> xs;
    PtrPack<uint8_t *> cs;
    PtrPack<float *> ss;
    for (int k = 0; k < K; ++k) {
        if (!codes_out_host[k] || !scales_out_host[k]) return DLCX_EINVAL;
        if (!aligned16(codes_out_host[k]) || !aligned16(scales_out_host[k])) return DLCX_EINVAL;
        factors[k] = reinterpret_cast<float *>(workspace) + (int64_t)k * count;
        xs.p[k] = factors[k];
        cs.p[k] = codes_out_host[k];
        ss.p[k] = scales_out_host[k];
    }
    void *inner = reinterpret_cast<char *>(workspace) + factor_region_bytes(desc, K);
    rc = dlcx_project(desc, phase, K, deltas_host, basis, factors, inner, stream);
    if (rc != DLCX_OK) return rc;
    return launch_quantize(K, xs, count, desc->qbits, desc->group, cs, ss, as_stream(stream));
}

int dlcx_compress(const dlcx_desc *desc, int phase, const float *delta, const float *basis,
                  uint8_t *codes_out, float *scales_out, void *workspace, void *stream) {
    const float *d[1] = {delta};
    uint8_t *c[1] = {codes_out};
    float *s[1] = {scales_out};
    return dlcx_compress_batched(desc, phase, 1, d, basis, c, s, workspace, stream);
}

int dlcx_dequant_average(int K, const uint8_t *const *codes_host, const float *const *scales_host,
                         int64_t count, int qbits, int group, float *mean_out, void *stream) {
    if (K < 1 || K > DLCX_MAX_WORKERS || count < 0 || (qbits != 4 && qbits != 8) ||
        !group_ok(group) || count % group)
        return DLCX_EINVAL;
    if (count == 0) return DLCX_OK;
    if (!codes_host || !scales_host || !mean_out || !aligned16(mean_out)) return DLCX_EINVAL;
    PtrPack<const uint8_t *> cs;
    PtrPack<const float *> ss;
    for (int k = 0; k < K; ++k) {
        if (!codes_host[k] || !scales_host[k]) return DLCX_EINVAL;
        if (!aligned16(codes_host[k]) || !aligned16(scales_host[k])) return DLCX_EINVAL;
        cs.p[k] = codes_host[k];
        ss.p[k] = scales_host[k];
    }
    return launch_dequant_average(K, cs, ss, count, qbits, group, mean_out, as_stream(stream));
}

int dlcx_orthonormalize(int64_t L, int32_t r, float *p_inout, void *workspace, void *stream) {
    if (L <= 0 || L % 16 || r < 1 || r > DLCX_MAX_RANK || r > L) return DLCX_EINVAL;
    if (!p_inout || !workspace || !aligned16(p_inout) || !aligned16(workspace)) return DLCX_EINVAL;
    return launch_orthonormalize(L, r, p_inout, workspace, as_stream(stream));
}

int dlcx_average(const dlcx_desc *desc, int phase, int K, const uint8_t *const *codes_host,
                 const float *const *scales_host, float *factor_out, void *workspace,
                 void *stream) {
    int rc = check_desc(desc);
    if (rc != DLCX_OK) return rc;
    if (phase != DLCX_PHASE_P && phase != DLCX_PHASE_Q) return DLCX_EINVAL;
    const int64_t L = phase == DLCX_PHASE_P ? desc->m : desc->n;
    rc = dlcx_dequant_average(K, codes_host, scales_host, (int64_t)desc->r * L, desc->qbits,
                              desc->group, factor_out, stream);
    if (rc != DLCX_OK || phase == DLCX_PHASE_Q) return rc;
    return dlcx_orthonormalize(L, desc->r, factor_out, workspace, stream);
}

// ---- dlcx_average without a workspace argument and without any allocation -----------------
// The scratch of the orthonormalisation in the library's own device image.  In host code the
// array's name is only a handle: the device address comes from hipGetSymbolAddress, once per
// device with that device current, and only that address is ever handed to a kernel.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices];  // per device, nullptr until first use there

static int static_scratch_ptr(void **out) {
    int dev = -1;
    int rc = note_hip(hipGetDevice(&dev), "static scratch: current device");
    if (rc != DLCX_OK) return rc;
    if (dev < 0 || dev >= kMaxDevices) return DLCX_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        rc = note_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "static scratch: address");
        if (rc != DLCX_OK) return rc;
        if (!ptr) return DLCX_ELAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return DLCX_OK;
}

size_t dlcx_static_scratch_bytes(void) { return kStaticScratchBytes; }

size_t dlcx_static_scratch_need(const dlcx_desc *desc, int phase) {
    if (check_desc(desc) != DLCX_OK || phase != DLCX_PHASE_P) return 0;
    return orth_workspace_bytes(desc->m, desc->r);
}

int dlcx_average_static(const dlcx_desc *desc, int phase, int K, const uint8_t *const *codes_host,
                        const float *const *scales_host, float *factor_out, void *stream) {
    int rc = check_desc(desc);
    if (rc != DLCX_OK) return rc;
    if (phase != DLCX_PHASE_P && phase != DLCX_PHASE_Q) return DLCX_EINVAL;
    // everything dlcx_average would reject is rejected here, before the runtime is touched
    if (K < 1 || K > DLCX_MAX_WORKERS || !codes_host || !scales_host || !factor_out ||
        !aligned16(factor_out))
        return DLCX_EINVAL;
    for (int k = 0; k < K; ++k)
        if (!codes_host[k] || !scales_host[k] || !aligned16(codes_host[k]) ||
            !aligned16(scales_host[k]))
            return DLCX_EINVAL;
    if (dlcx_static_scratch_need(desc, phase) > kStaticScratchBytes) return DLCX_ETOOBIG;
    void *ws = nullptr;
    if (phase == DLCX_PHASE_P) {
        rc = static_scratch_ptr(&ws);
        if (rc != DLCX_OK) return rc;
    }
    return dlcx_average(desc, phase, K, codes_host, scales_host, factor_out, ws, stream);
}

static int decompress_common(const dlcx_desc *desc, const float *p_hat, const float *q_bar,
                             float *delta_hat_out, int K, float *const *ef_inout_host,
                             const void *const *theta_l_host, int theta_l_dtype, float *theta,
                             float *vel, int apply, float lr, float mu, void *workspace,
                             void *stream) {
    int rc = check_desc(desc);
    if (rc != DLCX_OK) return rc;
    if (K < 0 || K > DLCX_MAX_WORKERS || !p_hat || !q_bar) return DLCX_EINVAL;
    if (K > 0 && !ef_inout_host) return DLCX_EINVAL;
    if (!aligned16(p_hat) || !aligned16(q_bar) || !aligned16(delta_hat_out) ||
        !aligned16(workspace))
        return DLCX_EINVAL;
    if (reconstruct_workspace_bytes(desc->mma, desc->m, desc->n, desc->r) > 0 && !workspace)
        return DLCX_EINVAL;
    ReconEpilogue ep;
    memset(&ep, 0, sizeof ep);
    ep.out = delta_hat_out;
    ep.K = K;
    ep.theta = theta;
    ep.vel = vel;
    ep.apply = apply;
    ep.lr = lr;
    ep.mu = mu;
    if (theta_l_host) {
        if (theta_l_dtype != DLCX_F32 && theta_l_dtype != DLCX_BF16) return DLCX_EINVAL;
        ep.tl_on = 1;
        ep.tl_bf16 = theta_l_dtype == DLCX_BF16;
    }
    if ((ep.tl_on || apply) && (!theta || !aligned16(theta))) return DLCX_EINVAL;
    if (apply && (!vel || !aligned16(vel) || !(lr == lr) || !(mu == mu))) return DLCX_EINVAL;
    if (K == 0 && !delta_hat_out && !apply) return DLCX_OK;
    for (int k = 0; k < K; ++k) {
        if (!ef_inout_host[k] || !aligned16(ef_inout_host[k])) return DLCX_EINVAL;
        ep.ef.p[k] = ef_inout_host[k];
        if (ep.tl_on) {
            if (!theta_l_host[k] || !aligned16(theta_l_host[k])) return DLCX_EINVAL;
            ep.tl.p[k] = theta_l_host[k];
        }
    }
    return launch_reconstruct(desc->mma, desc->m, desc->n, desc->r, p_hat, q_bar, ep, workspace,
                              as_stream(stream));
}

int dlcx_decompress(const dlcx_desc *desc, const float *p_hat, const float *q_bar,
                    float *delta_hat_out, int K, float *const *ef_inout_host, void *workspace,
                    void *stream) {
    return decompress_common(desc, p_hat, q_bar, delta_hat_out, K, ef_inout_host, nullptr, 0,
                             nullptr, nullptr, 0, 0.f, 0.f, workspace, stream);
}

int dlcx_decompress_apply(const dlcx_desc *desc, const float *p_hat, const float *q_bar, int K,
                          float *const *ef_inout_host, float *theta_g, float *v, float lr,
                          float mu, void *workspace, void *stream) {
    return decompress_common(desc, p_hat, q_bar, nullptr, K, ef_inout_host, nullptr, 0, theta_g, v,
                             1, lr, mu, workspace, stream);
}

int dlcx_ef_delta_apply(const dlcx_desc *desc, const float *p_hat, const float *q_bar, int K,
                        const void *const *theta_l_host, int theta_l_dtype,
                        float *const *ef_inout_host, float *theta_g, float *v, float lr, float mu,
                        void *workspace, void *stream) {
    if (K < 1 || !theta_l_host) return DLCX_EINVAL;
    return decompress_common(desc, p_hat, q_bar, nullptr, K, ef_inout_host, theta_l_host,
                             theta_l_dtype, theta_g, v, 1, lr, mu, workspace, stream);
}

int dlcx_ef_delta_apply_compress(const dlcx_desc *desc, int32_t r_prev, const float *p_hat,
                                 const float *q_bar, int K, const void *const *theta_l_host,
                                 int theta_l_dtype, float *const *ef_inout_host, float *theta_g,
                                 float *v, float lr, float mu, const float *basis,
                                 uint8_t *const *codes_out_host, float *const *scales_out_host,
                                 void *workspace, void *stream) {
    int rc = check_desc(desc);
    if (rc != DLCX_OK) return rc;
    if (r_prev < 0 || r_prev > DLCX_MAX_RANK || r_prev > desc->m || r_prev > desc->n)
        return DLCX_EINVAL;
    if (K < 1 || K > DLCX_MAX_WORKERS || !theta_l_host || !ef_inout_host || !theta_g || !basis ||
        !codes_out_host || !scales_out_host || !workspace)
        return DLCX_EINVAL;
    if (theta_l_dtype != DLCX_F32 && theta_l_dtype != DLCX_BF16) return DLCX_EINVAL;
    if (!aligned16(theta_g) || !aligned16(basis) || !aligned16(workspace)) return DLCX_EINVAL;
    if (r_prev > 0) {
        if (!p_hat || !q_bar || !v || !aligned16(p_hat) || !aligned16(q_bar) || !aligned16(v))
            return DLCX_EINVAL;
        if (!(lr == lr) || !(mu == mu)) return DLCX_EINVAL;
    }
    for (int k = 0; k < K; ++k) {
        if (!theta_l_host[k] || !ef_inout_host[k] || !codes_out_host[k] || !scales_out_host[k])
            return DLCX_EINVAL;
        if (!aligned16(theta_l_host[k]) || !aligned16(ef_inout_host[k]) ||
            !aligned16(codes_out_host[k]) || !aligned16(scales_out_host[k]))
            return DLCX_EINVAL;
    }
    // No fused kernel in the FMA mode.  Above rank 64 the fused kernel needs a launch per two
    // workers (ranks up to 128; its accumulators are r x 32 per worker and wavefront) or per
    // worker (above), each launch reconstructing the previous average again and re-reading the
    // fragments of both products; the feedback / update sweep followed by the projection kernel
    // moves 16 more bytes per element and is faster there (measured at ranks 96 and 128 on the
    // benchmark shapes with two workers per launch: 0.91 against 1.30 ms for an 8192 x 8192
    // matrix with four workers, 3.45 against 4.30 ms for 8192 x 28672).  Dealing the rank out over
    // the wavefronts instead (one launch for four workers, delta tiles exchanged through LDS) was
    // measured too: 1.74 against 1.27 + 0.40 ms per matrix at rank 187, its matrix-core phases
    // run with no loads of that workgroup in flight.
    if (desc->mma == DLCX_MMA_FMA || desc->r > 64) {
        if (r_prev > 0) {
            dlcx_desc dp = *desc;
            dp.r = r_prev;
            rc = dlcx_ef_delta_apply(&dp, p_hat, q_bar, K, theta_l_host, theta_l_dtype,
                                     ef_inout_host, theta_g, v, lr, mu, workspace, stream);
            if (rc != DLCX_OK) return rc;
        } else {
            for (int k = 0; k < K; ++k) {
                rc = dlcx_delta_ef(theta_g, theta_l_host[k], theta_l_dtype, ef_inout_host[k],
                                   desc->m * desc->n, stream);
                if (rc != DLCX_OK) return rc;
            }
        }
        return dlcx_compress_batched(desc, DLCX_PHASE_P, K, ef_inout_host, basis, codes_out_host,
                                     scales_out_host, workspace, stream);
    }
    const int64_t count = (int64_t)desc->r * desc->m;
    ReconEpilogue ep;
    memset(&ep, 0, sizeof ep);
    ep.K = K;
    ep.tl_on = 1;
    ep.tl_bf16 = theta_l_dtype == DLCX_BF16;
    ep.theta = theta_g;
    ep.vel = v;
    ep.apply = r_prev > 0;
    ep.lr = lr;
    ep.mu = mu;
    PtrPack<float *> factors;
    PtrPack<const float *> xs;
    PtrPack<uint8_t *> cs;
    PtrPack<float *> ss;
    for (int k = 0; k < K; ++k) {
        ep.ef.p[k] = ef_inout_host[k];
        ep.tl.p[k] = theta_l_host[k];
        factors.p[k] = reinterpret_cast<float *>(workspace) + (int64_t)k * count;
        xs.p[k] = factors.p[k];
        cs.p[k] = codes_out_host[k];
        ss.p[k] = scales_out_host[k];
    }
    void *inner = reinterpret_cast<char *>(workspace) + factor_region_bytes(desc, K);
    rc = launch_round_mfma(desc->mma, desc->m, desc->n, desc->r, r_prev, p_hat, q_bar, basis, ep,
                           factors, inner, as_stream(stream));
    if (rc != DLCX_OK) return rc;
    return launch_quantize(K, xs, count, desc->qbits, desc->group, cs, ss, as_stream(stream));
}

int dlcx_effective_rank(int64_t L, int32_t r, const float *q_bar, double tau,
                        int32_t *rprime_out_dev, void *workspace, void *stream) {
    if (L <= 0 || L % 16 || r < 1 || r > DLCX_MAX_RANK || r > L) return DLCX_EINVAL;
    if (!(tau > 0.0 && tau <= 1.0)) return DLCX_EINVAL;
    if (!q_bar || !rprime_out_dev || !workspace || !aligned16(q_bar) || !aligned16(workspace))
        return DLCX_EINVAL;
    return launch_effective_rank(L, r, q_bar, tau, rprime_out_dev, workspace, as_stream(stream));
}

size_t dlcx_batched_workspace_bytes(const dlcx_desc *descs_host, int n_matrices) {
    if (n_matrices < 0 || (n_matrices > 0 && !descs_host)) return 0;
    size_t total = 0;
    for (int i = 0; i < n_matrices; ++i) {
        if (check_desc(&descs_host[i]) != DLCX_OK) return 0;
        const size_t a = orth_workspace_bytes(descs_host[i].m, descs_host[i].r);
        const size_t b = effrank_workspace_bytes(descs_host[i].n, descs_host[i].r);
        total += a > b ? a : b;
    }
    return total;
}

int dlcx_orthonormalize_batched(const dlcx_desc *descs_host, float *const *p_inout_host,
                                int n_matrices, void *workspace, void *stream) {
    if (n_matrices < 0) return DLCX_EINVAL;
    if (n_matrices == 0) return DLCX_OK;
    if (!descs_host || !p_inout_host || !workspace || !aligned16(workspace)) return DLCX_EINVAL;
    for (int i = 0; i < n_matrices; ++i) {
        if (check_desc(&descs_host[i]) != DLCX_OK) return DLCX_EINVAL;
        if (!p_inout_host[i] || !aligned16(p_inout_host[i])) return DLCX_EINVAL;
    }
    char *ws = reinterpret_cast<char *>(workspace);
    for (int i0 = 0; i0 < n_matrices; i0 += kMaxBatch) {
        FactorBatch b;
        b.n = n_matrices - i0 < kMaxBatch ? n_matrices - i0 : kMaxBatch;
        for (int i = 0; i < b.n; ++i) {
            const dlcx_desc &d = descs_host[i0 + i];
            orth_item(&b.it[i], p_inout_host[i0 + i], d.m, d.r, ws);
            b.it[i].out = nullptr;
            ws += orth_workspace_bytes(d.m, d.r);
        }
        int rc = launch_orthonormalize_batch(b, as_stream(stream));
        if (rc != DLCX_OK) return rc;
    }
    return DLCX_OK;
}

int dlcx_effective_rank_batched(const dlcx_desc *descs_host, const float *const *q_bars_host,
                                int n_matrices, double tau, int32_t *rprime_out_dev,
                                void *workspace, void *stream) {
    if (n_matrices < 0) return DLCX_EINVAL;
    if (n_matrices == 0) return DLCX_OK;
    if (!descs_host || !q_bars_host || !rprime_out_dev || !workspace || !aligned16(workspace))
        return DLCX_EINVAL;
    if (!(tau > 0.0 && tau <= 1.0)) return DLCX_EINVAL;
    for (int i = 0; i < n_matrices; ++i) {
        if (check_desc(&descs_host[i]) != DLCX_OK) return DLCX_EINVAL;
        if (!q_bars_host[i] || !aligned16(q_bars_host[i])) return DLCX_EINVAL;
    }
    char *ws = reinterpret_cast<char *>(workspace);
    for (int i0 = 0; i0 < n_matrices; i0 += kMaxBatch) {
        FactorBatch b;
        b.n = n_matrices - i0 < kMaxBatch ? n_matrices - i0 : kMaxBatch;
        for (int i = 0; i < b.n; ++i) {
            const dlcx_desc &d = descs_host[i0 + i];
            effrank_item(&b.it[i], q_bars_host[i0 + i], d.n, d.r, rprime_out_dev + i0 + i, ws);
            ws += effrank_workspace_bytes(d.n, d.r);
        }
        int rc = launch_effective_rank_batch(b, tau, as_stream(stream));
        if (rc != DLCX_OK) return rc;
    }
    return DLCX_OK;
}

static int window_rule(int32_t rprime, int32_t *hist, int32_t t, int32_t c, int32_t r1,
                       int32_t rmin, int32_t rmax, int32_t H1, int32_t *r_next, int32_t *H_next) {
    hist[(t - 1) % c] = rprime;
    if (t < c) {
        *r_next = r1;
        *H_next = H1;
        return DLCX_OK;
    }
    int64_t sum = 0;
    for (int i = 0; i < c; ++i) sum += hist[i];
    int64_t rt = (2 * sum + c) / (2 * (int64_t)c);
    if (rt < rmin) rt = rmin;
    if (rt > rmax) rt = rmax;
    // H_t = H_1 (r_1 - r_t) / r_1, rounded half-up, at least 1
    const int64_t num = (int64_t)H1 * ((int64_t)r1 - rt);
    int64_t H = num >= 0 ? (2 * num + r1) / (2 * (int64_t)r1) : 0;
    if (H < 1) H = 1;
    *r_next = (int32_t)rt;
    *H_next = (int32_t)H;
    return DLCX_OK;
}

int dlcx_select_rank_from(const int32_t *rprime_dev, int n_matrices, int32_t *rprime_hist_host,
                          int32_t t, int32_t c, int32_t r1, int32_t rmin, int32_t rmax, int32_t H1,
                          int32_t *rprime_inout_host, int32_t *r_next_out_host,
                          int32_t *H_next_out_host, void *stream) {
    if (n_matrices < 0 || t < 1 || c < 1 || r1 < 1 || rmin < 1 || rmax < rmin || H1 < 1)
        return DLCX_EINVAL;
    if (!rprime_hist_host || !rprime_inout_host || !r_next_out_host || !H_next_out_host)
        return DLCX_EINVAL;
    if (n_matrices > 0) {
        if (!rprime_dev) return DLCX_EINVAL;
        std::vector<int32_t> vals((size_t)n_matrices);
        int rc = note_hip(hipMemcpyAsync(vals.data(), rprime_dev, vals.size() * sizeof(int32_t),
                                         hipMemcpyDeviceToHost, as_stream(stream)),
                          "select_rank copy");
        if (rc != DLCX_OK) return rc;
        rc = note_hip(hipStreamSynchronize(as_stream(stream)), "select_rank sync");
        if (rc != DLCX_OK) return rc;
        int64_t sum = 0;
        for (int i = 0; i < n_matrices; ++i) sum += vals[i] > 0 ? vals[i] : rmin;
        *rprime_inout_host = (int32_t)((2 * sum + n_matrices) / (2 * (int64_t)n_matrices));
    }
    return window_rule(*rprime_inout_host, rprime_hist_host, t, c, r1, rmin, rmax, H1,
                       r_next_out_host, H_next_out_host);
}

int dlcx_select_rank(const dlcx_desc *descs_host, const float *const *q_bars_host, int n_matrices,
                     double tau, int32_t *rprime_hist_host, int32_t t, int32_t c, int32_t r1,
                     int32_t rmin, int32_t rmax, int32_t H1, int32_t *rprime_inout_host,
                     int32_t *r_next_out_host, int32_t *H_next_out_host, void *workspace,
                     void *stream) {
    if (n_matrices < 0) return DLCX_EINVAL;
    int32_t *out_dev = nullptr;
    if (n_matrices > 0) {
        if (!descs_host || !q_bars_host || !workspace || !aligned16(workspace)) return DLCX_EINVAL;
        if (!(tau > 0.0 && tau <= 1.0)) return DLCX_EINVAL;
        if (t < 1 || c < 1 || r1 < 1 || rmin < 1 || rmax < rmin || H1 < 1 || !rprime_hist_host ||
            !rprime_inout_host || !r_next_out_host || !H_next_out_host)
            return DLCX_EINVAL;
        for (int i = 0; i < n_matrices; ++i) {
            if (check_desc(&descs_host[i]) != DLCX_OK) return DLCX_EINVAL;
            if (!q_bars_host[i] || !aligned16(q_bars_host[i])) return DLCX_EINVAL;
        }
        out_dev = reinterpret_cast<int32_t *>(workspace);
        char *ws = reinterpret_cast<char *>(workspace) + align256((size_t)n_matrices * sizeof(int32_t));
        int rc = dlcx_effective_rank_batched(descs_host, q_bars_host, n_matrices, tau, out_dev, ws,
                                             stream);
        if (rc != DLCX_OK) return rc;
    }
    return dlcx_select_rank_from(out_dev, n_matrices, rprime_hist_host, t, c, r1, rmin, rmax, H1,
                                 rprime_inout_host, r_next_out_host, H_next_out_host, stream);
}

}  // extern "C"
