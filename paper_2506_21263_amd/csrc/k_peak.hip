// Measurement aid, not a step of the method: the rate at which this GPU retires
// v_mfma_f32_32x32x16_bf16 when nothing else competes.  Every wavefront keeps 8 independent
// accumulator tiles and issues `iters` rounds of 8 MFMAs on fixed operands; the sum of the
// accumulators is written out so that the work cannot be removed.  The result is the
// denominator for "fraction of the attainable matrix-core rate" beside the datasheet peak.
#include "common.h"

namespace dlcx {

typedef __bf16 pk_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pk_f32x16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, float *__restrict__ out) {
    pk_f32x16 acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
    pk_bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((threadIdx.x + e) & 3);
        b[e] = (__bf16)(float)((threadIdx.x * 3 + e) & 1);
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < 8; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[t][v];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

int launch_mfma_peak(int workgroups, int iters, float *out, hipStream_t st) {
    Timed timed(KID_MFMA_PEAK, st);
    hipLaunchKernelGGL(mfma_peak_kernel, dim3((unsigned)workgroups), dim3(256), 0, st, iters, out);
    return check_launch("mfma_peak");
}

}  // namespace dlcx
