/*
 * dlcx -- the per-stage outer step of DiLoCoX (arXiv 2506.21263) on one MI355X.
 *
 * C ABI of libdlcx_hip.so.  Every pointer is a DEVICE pointer unless its name
 * ends in _host; arrays of pointers (one entry per simulated data-parallel
 * worker) are HOST arrays of device pointers.  The library keeps no state and
 * never allocates device memory: the caller owns every buffer, scratch space is passed as
 * `workspace` (size from dlcx_workspace_bytes).  All calls are asynchronous on
 * `stream` (a hipStream_t, NULL = the default stream) and never synchronise,
 * except dlcx_select_rank, which returns integers to the host.
 *
 * Layout
 *   matrix  : m x n, row-major fp32, element (i, j) at i*n + j.
 *   factor  : P is m x r, Q is n x r; stored column by column, column c of a
 *             factor of length L at c*L .. c*L+L  (so a factor is an r x L
 *             row-major array).  The basis passed to the P phase is Q_in
 *             (r x n), the basis of the Q phase is P_hat (r x m).
 *   payload : codes + scales of one quantised factor.  Groups are `group`
 *             consecutive elements of one factor column, one fp32 scale per
 *             group.  int8: one signed byte per element.  int4: element 2j in
 *             the low nibble of byte j, element 2j+1 in the high nibble,
 *             two's complement.
 *   All buffers must be 16-byte aligned.
 *
 * Errors: every function returns 0 (DLCX_OK) or a negative code; arguments
 * are validated on the host before anything is launched, so a failed call
 * has launched nothing.
 *
 * Determinism: no floating-point atomics; the same inputs give bitwise the
 * same outputs from run to run.
 */
#ifndef DLCX_H
#define DLCX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DLCX_OK 0
#define DLCX_EINVAL (-1)       /* NULL/misaligned pointer, shape or parameter out of range */
#define DLCX_EUNSUPPORTED (-2) /* valid request this build has no kernel for              */
#define DLCX_ELAUNCH (-3)      /* the HIP runtime reported an error                       */
#define DLCX_ETOOBIG (-4)      /* larger than the fixed scratch of an entry point that does
                                  not allocate (dlcx_average_static)                      */

#define DLCX_MAX_RANK 256
#define DLCX_MAX_WORKERS 16

enum { DLCX_PHASE_P = 0, DLCX_PHASE_Q = 1 };
enum { DLCX_F32 = 0, DLCX_BF16 = 1 };
/* arithmetic of the three rank-r products (projections and reconstruction) */
enum {
    DLCX_MMA_FMA = 0,  /* fp32 operands, fp64 accumulation on the vector ALU                   */
    DLCX_MMA_F32 = 1,  /* fp32-accurate on the bf16 matrix cores: operands split into three
                          bf16 pieces, six piece products, fp32 accumulation (rel-L2 <= 1e-5) */
    DLCX_MMA_BF16 = 2, /* bf16 matrix cores, operands split into two bf16 pieces, three piece
                          products, fp32 accumulation (rel-L2 <= 2e-3 with a wide margin)     */
    DLCX_MMA_F16 = 3   /* as DLCX_MMA_BF16, except the two projections at ranks above 64 (where
                          the matrix cores, not the stream of delta, set the pace): there one
                          fp16 product per block, operands scaled by exact powers of two into
                          fp16's range, fp32 accumulation (rel-L2 <= 2e-3, measured 2e-5 .. 4e-4).
                          A launch whose largest |delta| lies outside [2^-14, 15.99) is redone
                          in the DLCX_MMA_BF16 arithmetic by a stand-by launch, without a
                          synchronisation; the result never depends on fp16's range             */
};

typedef struct {
    int64_t m, n;   /* matrix shape; m % group == 0 and n % group == 0            */
    int32_t r;      /* rank, 1 <= r <= min(m, n, DLCX_MAX_RANK)                   */
    int32_t qbits;  /* 4 or 8                                                     */
    int32_t group;  /* quantisation group: 16, 32, 64, 128 or 256                 */
    int32_t mma;    /* DLCX_MMA_*                                                 */
} dlcx_desc;

/* Pseudo-gradient with error compensation (Alg. 2; Appendix A.3, first display):
 *   ef_inout[x] <- (theta_g[x] - theta_l[x]) + ef_inout[x]
 * ef_inout holds the error buffer e_i on entry and delta_i on return.  theta_l is fp32
 * (DLCX_F32) or bf16 (DLCX_BF16).  numel >= 0. */
int dlcx_delta_ef(const float *theta_g, const void *theta_l, int theta_l_dtype,
                  float *ef_inout, int64_t numel, void *stream);

/* Compressor C[delta] of Alg. 1 for one worker and one phase of the shared-basis low-rank
 * step: phase P computes P_i = delta * Q_in (basis = Q_in, r x n), phase Q computes
 * Q_i = delta^T * P_hat (basis = P_hat, r x m); the factor is then quantised to
 * qbits in groups.  On return the first r*L floats of `workspace` hold the fp32 factor
 * that was quantised (L = m for phase P, n for phase Q). */
int dlcx_compress(const dlcx_desc *desc, int phase, const float *delta, const float *basis,
                  uint8_t *codes_out, float *scales_out, void *workspace, void *stream);

/* The same for K workers in one launch sequence (deltas_host[k], codes_out_host[k],
 * scales_out_host[k]); the workspace then holds K factors back to back. */
int dlcx_compress_batched(const dlcx_desc *desc, int phase, int K,
                          const float *const *deltas_host, const float *basis,
                          uint8_t *const *codes_out_host, float *const *scales_out_host,
                          void *workspace, void *stream);

/* The AllReduce-average of Alg. 2 over the K data-parallel workers, on payloads held in this
 * GPU's memory: factor_out = (1/K) sum_k dequant(codes_k, scales_k), workers added in index
 * order.  For phase P the mean is then orthonormalised in place (see dlcx_orthonormalize),
 * giving P_hat; for phase Q the mean Q_bar is returned as is. */
int dlcx_average(const dlcx_desc *desc, int phase, int K, const uint8_t *const *codes_host,
                 const float *const *scales_host, float *factor_out, void *workspace,
                 void *stream);

/* dlcx_average for callers that cannot allocate device memory and cannot hand in a workspace
 * either: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and bitwise the same result as dlcx_average, but the scratch of
 * the orthonormalisation (phase P) lives in a fixed array inside the library's device image:
 * dlcx_static_scratch_bytes() bytes (32 MiB) per GPU the library runs on, held until the process
 * ends.  A factor whose orthonormalisation needs more (dlcx_static_scratch_need reports the need;
 * r = 256 fits up to m = 31232, r = 64 up to m = 522752) is rejected with DLCX_ETOOBIG before
 * anything is launched.  The call allocates nothing, frees nothing and does not synchronise.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two host threads) race on it and must be ordered by the caller; nothing in the array
 * has to survive from one call to the next and nothing has to be cleared. */
int dlcx_average_static(const dlcx_desc *desc, int phase, int K, const uint8_t *const *codes_host,
                        const float *const *scales_host, float *factor_out, void *stream);
size_t dlcx_static_scratch_bytes(void);
/* Scratch bytes dlcx_average_static needs for this descriptor and phase (0 for phase Q and for a
 * bad descriptor). */
size_t dlcx_static_scratch_need(const dlcx_desc *desc, int phase);

/* Decompression Delta_hat = P_hat * Q_bar^T and the error buffer of Alg. 2,
 * e_i <- delta_i - Delta_hat, for K >= 0 workers.  delta_hat_out (m x n) may be NULL when only
 * the error buffers are wanted; ef_inout_host may be NULL when K == 0. */
int dlcx_decompress(const dlcx_desc *desc, const float *p_hat, const float *q_bar,
                    float *delta_hat_out, int K, float *const *ef_inout_host, void *workspace,
                    void *stream);

/* The same decompression fused with its two consumers in Alg. 2, so that Delta_hat is never
 * written to memory: e_i <- delta_i - Delta_hat for K >= 0 workers, then the OuterOpt step
 * v <- mu v + Delta_hat ; theta_g <- theta_g - lr (Delta_hat + mu v), all tile by tile. */
int dlcx_decompress_apply(const dlcx_desc *desc, const float *p_hat, const float *q_bar, int K,
                          float *const *ef_inout_host, float *theta_g, float *v, float lr,
                          float mu, void *workspace, void *stream);

/* One pass over the matrix for everything Alg. 2 does between two compressions (outer step
 * t >= 2), in its order:  e_i <- delta_i - Delta_hat  (previous round's average, P_hat Q_bar^T,
 * never written to memory);  delta_i <- (theta_g - theta_l,i) + e_i  with theta_g still the
 * value of step t-1;  then  theta_g <- OuterOpt(theta_g, Delta_hat).  The same steps as
 * dlcx_decompress (error buffers), K x dlcx_delta_ef and dlcx_outer_nesterov in that order, equal
 * to them up to fp32 rounding and not bit for bit: dlcx_delta_ef evaluates (theta_g - theta_l) + e
 * in fp64 and rounds once, this pass rounds theta_g - theta_l, delta_i - Delta_hat and their sum
 * to fp32 one after the other (at most one unit in the last place of each apart). */
int dlcx_ef_delta_apply(const dlcx_desc *desc, const float *p_hat, const float *q_bar, int K,
                        const void *const *theta_l_host, int theta_l_dtype,
                        float *const *ef_inout_host, float *theta_g, float *v, float lr, float mu,
                        void *workspace, void *stream);

/* dlcx_ef_delta_apply followed by the P phase of dlcx_compress_batched, with the new
 * pseudo-gradients read once for both: while a tile of delta_i is on chip it is also multiplied
 * with the basis Q_in (r x n), so P_i = delta_i Q_in costs no second sweep over the matrix.
 * desc->r is the rank of the compression that starts; r_prev the rank of p_hat / q_bar
 * (r_prev == 0: outer step 1, there is no previous average: only delta_i <- (theta_g -
 * theta_l,i) + e_i and the projection; p_hat, q_bar and v are then unused).  On return the
 * workspace starts with the K fp32 factors, as after dlcx_compress_batched.  The workspace must
 * be sized (dlcx_workspace_bytes) for a descriptor whose r is the larger of the two ranks.
 * Which arithmetic forms delta_i depends on the path taken: the one-sweep kernel (MFMA modes,
 * desc->r <= 64) and dlcx_ef_delta_apply (MFMA modes above that rank, and the FMA mode with
 * r_prev > 0) use the three fp32 roundings described there; the FMA mode at r_prev == 0 calls
 * dlcx_delta_ef (fp64 sum, one rounding).  The last bit of delta_i may therefore differ between
 * paths; every path is within the mode's tolerance of the oracle, which follows dlcx_delta_ef. */
int dlcx_ef_delta_apply_compress(const dlcx_desc *desc, int32_t r_prev, const float *p_hat,
                                 const float *q_bar, int K, const void *const *theta_l_host,
                                 int theta_l_dtype, float *const *ef_inout_host, float *theta_g,
                                 float *v, float lr, float mu, const float *basis,
                                 uint8_t *const *codes_out_host, float *const *scales_out_host,
                                 void *workspace, void *stream);

/* Outer step t of Alg. 2 for one tensor whose compressor is the quantiser alone: Alg. 1 with
 * the LOWRANK step left out, C(delta) = QUANTIZE(delta | q), the Int4-only setting the paper
 * reports for its smaller model (Sec. 4.1) and the only form that applies to tensors that are
 * not matrices.  The tensor is `numel` consecutive elements (a multiple of `group`); a group is
 * `group` consecutive elements.  In the order of Alg. 2, in one sweep:
 *   Delta^{t-1} = mean_k dequant(prev payload_k), workers in index order; with requant != 0
 *                 re-encoded to q bits first (what a q-bit reduction would hand on);
 *   e_k <- delta_k - Delta^{t-1} ;  delta_k <- (theta_g - theta_l,k) + e_k   (in place over
 *                 ef_inout_host[k], theta_g still the value of step t-1);
 *   payload_k <- QUANTIZE(delta_k) into codes_out_host[k] / scales_out_host[k];
 *   theta_g <- OuterOpt(theta_g, Delta^{t-1}), v likewise.
 * prev_codes_host == NULL is outer step 1: no feedback, no update, v is not touched.  The new
 * payload of a worker may be written over its previous one (codes_out_host[k] ==
 * prev_codes_host[k] and the same for the scales).  All pointer arrays are host arrays of K
 * device pointers; payload sizes are numel/2 (q = 4) or numel (q = 8) bytes of codes and
 * numel/group fp32 scales.  The averaged pseudo-gradient is never written to memory.  The mean,
 * the sum (theta_g - theta_l) + e and the OuterOpt step (lr, mu as doubles) are evaluated in
 * fp64 and rounded to fp32 once each; the results do not depend on the launch shape. */
int dlcx_quant_round(int64_t numel, int qbits, int group, int K,
                     const void *const *theta_l_host, int theta_l_dtype,
                     float *const *ef_inout_host, float *theta_g, float *v, double lr, double mu,
                     const uint8_t *const *prev_codes_host, const float *const *prev_scales_host,
                     int requant, uint8_t *const *codes_out_host, float *const *scales_out_host,
                     void *stream);

/* Error buffers of Alg. 2 against a materialised average: e_k <- delta_k - Delta for K workers,
 * in place, `numel` elements each. */
int dlcx_ef_update(int K, float *const *ef_inout_host, const float *delta_hat, int64_t numel,
                   void *stream);

/* x <- dequant(QUANTIZE(x | q)) in place on `count` floats in consecutive groups: an averaged
 * factor (or tensor) re-encoded to q bits, as a reduction that carries q-bit values between its
 * hops would deliver it, instead of the fp32 mean that dlcx_average leaves. */
int dlcx_requantize(float *x_inout, int64_t count, int qbits, int group, void *stream);

/* Measurement aid, not a step of the method: `workgroups` workgroups of 4 wavefronts each issue
 * 8 * iters independent v_mfma_f32_32x32x16_bf16 (32768 flop each); `out` (workgroups * 256
 * floats, device) receives the accumulator sums.  Timed with the profiler (kernel "mfma_peak"),
 * it gives the matrix-core rate this GPU attains when nothing competes.  operands = 0: every
 * operand element is a small integer (few bits toggle); operands = 1: pseudo-random signs,
 * exponents and mantissas, four operand pairs in rotation, which is what real data looks like to
 * the multipliers -- the rate is lower, because the clock follows the power drawn. */
int dlcx_mfma_peak_probe(int workgroups, int iters, int operands, float *out, void *stream);

/* Measurement aid, not a step of the method: the HBM traffic of one launch of the fused kernel
 * behind dlcx_ef_delta_apply_compress -- per element, K error buffers read and written, K
 * replicas read, theta_g and v read and written -- as a flat sweep: one 16-byte position of every
 * array per thread, workgroups in address order, no matrix-core work.  All K + 2 fp32 arrays are
 * OVERWRITTEN with sums of what was read, which mean nothing.  numel is a multiple of 1024.  Timed
 * with the profiler (kernel "traffic_probe"), it gives the rate the memory system reaches for
 * this mix of streams under the simplest access pattern, the yardstick for the fused kernel. */
int dlcx_traffic_probe(int K, const void *const *theta_l_host, int theta_l_dtype,
                       float *const *ef_inout_host, float *theta_g, float *v, int64_t numel,
                       void *stream);

/* Communication model of Sec. 2.4.1 (host only).  A ring all-reduce between `clusters` clusters
 * moves 2 (clusters - 1) / clusters of the payload over the link between two of them;
 * returns the seconds that takes at `bits_per_second`.  Negative on bad arguments. */
double dlcx_comm_seconds(double payload_bytes, int clusters, double bits_per_second);

/* Choice of (rank, local steps) that just hides the exchange of one outer step behind local
 * training (the one-step-delay overlap of Sec. 2.3 needs comm <= H * step time).  The payload
 * of a worker at rank r is power_iters times the sum over the n_matrices descriptors of both
 * quantised factors (r clipped to each matrix's smaller side; every power iteration of a round
 * sends both factors again, 1 in the paper) plus extra_bytes (tensors sent without low-rank).
 * *r_out is the largest rank in [rmin, rmax] whose exchange fits H * step_seconds and *H_out = H;
 * if not even rmin fits, *r_out = rmin and *H_out is the smallest H that hides it.
 * *comm_seconds_out is the exchange time at the chosen rank.  Host only. */
int dlcx_plan_overlap(const dlcx_desc *descs_host, int n_matrices, double extra_bytes,
                      int power_iters, int32_t rmin, int32_t rmax, int clusters,
                      double bits_per_second,
                      double step_seconds, int32_t H, int32_t *r_out, int32_t *H_out,
                      double *comm_seconds_out);

/* OuterOpt of Alg. 2 / Appendix A.3: SGD with Nesterov momentum on the averaged
 * pseudo-gradient,  v <- mu v + g ;  theta_g <- theta_g - lr (g + mu v).  In place. */
int dlcx_outer_nesterov(float *theta_g, float *v, const float *delta_hat, int64_t numel,
                        float lr, float mu, void *stream);

/* Alg. 3 (Adaptive Gradient Compress) for the outer step t that is about to compress.
 *   r'_t  : measured on the latest averages: per matrix, the smallest k whose k largest
 *           eigenvalues of Q_bar^T Q_bar hold at least tau of the trace; the stage value is
 *           the mean over the n_matrices matrices (a zero matrix counts as rmin), rounded
 *           half-up.  With n_matrices == 0 the value in *rprime_inout_host is used instead
 *           (the convention r'_1 = r_1 is the caller's).
 *   rule  : r'_t is stored in rprime_hist_host[(t-1) % c] (a caller-owned ring of c ints);
 *           t < c gives r_1 and H_1, otherwise r_t = mean of the ring, rounded half-up and
 *           clamped to [rmin, rmax], and H_t = max(1, round(H_1 (r_1 - r_t) / r_1)).
 * Synchronises `stream`.  workspace: dlcx_select_rank_workspace_bytes. */
int dlcx_select_rank(const dlcx_desc *descs_host, const float *const *q_bars_host,
                     int n_matrices, double tau, int32_t *rprime_hist_host, int32_t t,
                     int32_t c, int32_t r1, int32_t rmin, int32_t rmax, int32_t H1,
                     int32_t *rprime_inout_host, int32_t *r_next_out_host,
                     int32_t *H_next_out_host, void *workspace, void *stream);

/* The second half of dlcx_select_rank alone: the per-matrix r' values were already measured with
 * dlcx_effective_rank into the DEVICE array rprime_dev (n_matrices ints; with n_matrices == 0
 * the value in *rprime_inout_host is used).  Copies them back (synchronises `stream`), forms the
 * stage value and applies the window rule. */
int dlcx_select_rank_from(const int32_t *rprime_dev, int n_matrices, int32_t *rprime_hist_host,
                          int32_t t, int32_t c, int32_t r1, int32_t rmin, int32_t rmax, int32_t H1,
                          int32_t *rprime_inout_host, int32_t *r_next_out_host,
                          int32_t *H_next_out_host, void *stream);

/* ---- helpers: the steps the entry points above are made of ---------------------------- */

/* Size of one worker's payload for one factor: what Alg. 1 hands to the AllReduce of Alg. 2 is
 * the quantised FACTORS (Sec. 4.1: r_1 = 2048 is "about 2x" on a hidden-8192 model, i.e.
 * (m + n) r / (m n) = 0.5), r * L codes of qbits bits plus one fp32 scale per group.  Returns
 * codes + scales bytes (also through the two pointers, either may be NULL), 0 on a bad
 * descriptor.  Host only. */
size_t dlcx_payload_bytes(const dlcx_desc *desc, int phase, size_t *codes_bytes,
                          size_t *scales_bytes);
/* Device scratch needed by any per-matrix entry point above for this descriptor with up to K
 * workers (fp32 factors of Alg. 1 before quantisation, operand fragments, partial sums, the
 * fp64 scratch of the orthonormalisation and of Alg. 3's r').  0 on a bad descriptor.  Host only. */
size_t dlcx_workspace_bytes(const dlcx_desc *desc, int K);
/* Device scratch of dlcx_select_rank (Alg. 3) for these matrices.  Host only. */
size_t dlcx_select_rank_workspace_bytes(const dlcx_desc *descs_host, int n_matrices);

/* The LOWRANK step (1) of Alg. 1 alone, one of its two products for K workers:
 * factors_out_host[k] (r x L fp32) = delta_k * Q_in (phase P) or delta_k^T * P_hat (phase Q),
 * unquantised. */
int dlcx_project(const dlcx_desc *desc, int phase, int K, const float *const *deltas_host,
                 const float *basis, float *const *factors_out_host, void *workspace,
                 void *stream);
/* The QUANTIZE step (2) of Alg. 1 alone on `count` floats in consecutive groups: per group
 * scale = amax / qmax and code = clamp(rint(x * (qmax / amax))), qmax = 2^(qbits-1) - 1, round
 * half to even; a group whose amax is below 2^-100 gives scale 0 and codes 0. */
int dlcx_quantize(const float *x, int64_t count, int qbits, int group, uint8_t *codes_out,
                  float *scales_out, void *stream);
/* The AllReduce-average of Alg. 2 alone: mean_out = (1/K) sum_k dequant(codes_k, scales_k) over
 * `count` elements, workers added in index order (fp64 sum, one rounding), no
 * orthonormalisation. */
int dlcx_dequant_average(int K, const uint8_t *const *codes_host,
                         const float *const *scales_host, int64_t count, int qbits, int group,
                         float *mean_out, void *stream);
/* Orthonormalisation of the averaged P factor between the two products of Alg. 1's LOWRANK
 * step (the shared-basis power iteration the paper cites for it; the paper itself is silent on
 * the method).  Thin-QR Q-factor with positive diagonal of R of the L x r factor p_inout (r x L
 * storage), in place.  A column whose component orthogonal to the earlier columns is at most 1e-6 of
 * its norm (or that is zero) becomes the zero column. */
int dlcx_orthonormalize(int64_t L, int32_t r, float *p_inout, void *workspace, void *stream);
/* The orthonormalisation (Alg. 1, LOWRANK step) and the effective rank r' (Alg. 3's
 * "calculate r'_t with the averaged gradient") for ALL matrices of a stage at once (these
 * steps are short and latency-bound per matrix; batched, each matrix gets its own workgroups of
 * one launch).  Matrix i has shape descs_host[i]; p_inout_host[i] is its r x m factor,
 * q_bars_host[i] its r x n factor; rprime_out_dev receives n_matrices ints.  The workspace
 * (dlcx_batched_workspace_bytes) serves either call. */
size_t dlcx_batched_workspace_bytes(const dlcx_desc *descs_host, int n_matrices);
int dlcx_orthonormalize_batched(const dlcx_desc *descs_host, float *const *p_inout_host,
                                int n_matrices, void *workspace, void *stream);
int dlcx_effective_rank_batched(const dlcx_desc *descs_host, const float *const *q_bars_host,
                                int n_matrices, double tau, int32_t *rprime_out_dev,
                                void *workspace, void *stream);
/* Alg. 3's r'_t for one matrix (the paper gives no formula; see dlcx_select_rank for the
 * definition used): the smallest k whose k largest eigenvalues of Q_bar^T Q_bar hold at least
 * tau of the trace, written to a DEVICE int32 (0 when Q_bar is all zero); asynchronous. */
int dlcx_effective_rank(int64_t L, int32_t r, const float *q_bar, double tau,
                        int32_t *rprime_out_dev, void *workspace, void *stream);

/* ---- instrumentation ----------------------------------------------------------------------
 * Per-kernel timing with HIP events on the launch stream.  dlcx_profile_enable(1) clears the
 * records and starts recording every kernel launch of this library (process-wide; the records
 * are guarded by a lock, so launches from several host threads may be recorded at once, but
 * enabling or disabling while another thread launches loses that thread's launches in flight;
 * meant for benchmarks); dlcx_profile_read waits for the recorded launches of one
 * kernel id (0 .. dlcx_profile_kernels()-1) and returns their summed duration and count;
 * dlcx_profile_enable(0) stops recording and frees the events. */
int dlcx_profile_enable(int on);
int dlcx_profile_kernels(void);
const char *dlcx_profile_name(int kernel_id);
int dlcx_profile_read(int kernel_id, double *total_ms_host, int64_t *launches_host);

const char *dlcx_strerror(int code);
/* Text of the last HIP error seen by this thread's calls (empty if none). */
const char *dlcx_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DLCX_H */
