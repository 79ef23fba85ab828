// Measurement aid, not a step of the method: the rate at which this GPU retires
// v_mfma_f32_32x32x16_bf16 when nothing else competes.  Every wavefront keeps 8 independent
// accumulator tiles and issues `iters` rounds of 8 MFMAs on four operand pairs in rotation; the
// sum of the accumulators is written out so that the work cannot be removed.  With small-integer
// operands few bits toggle in the multipliers; with pseudo-random signs, exponents and mantissas
// (what real data looks like) the power drawn is higher and the clock, hence the rate, lower.
// The two results are the denominators for "fraction of the attainable matrix-core rate" beside
// the datasheet peak.
#include "common.h"

namespace dlcx {

typedef __bf16 pk_bf16x8 __attribute__((ext_vector_type(8)));
typedef float pk_f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t peak_hash(uint32_t x) {
    x ^= x >> 16;
    x *= 0x7feb352du;
    x ^= x >> 15;
    x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

// one bf16: random sign and mantissa, exponent 2^-10 .. 2^-1
__device__ __forceinline__ uint32_t peak_bf16(uint32_t h) {
    return ((h & 1u) << 15) | ((0x75u + ((h >> 1) % 10u)) << 7) | ((h >> 8) & 0x7fu);
}

__global__ __launch_bounds__(256) void mfma_peak_kernel(int iters, int operands,
                                                        float *__restrict__ out) {
    pk_f32x16 acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
    uint4 ar[4], br[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t w[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t seed = (uint32_t)threadIdx.x * 64u + (uint32_t)q * 8u + (uint32_t)e;
            if (operands == 0) {  // bf16 small integers: 0..3 and 0..1
                const uint32_t lo = ((threadIdx.x + e + q) & 3u), hi = ((threadIdx.x * 3 + e) & 1u);
                const __bf16 a0 = (__bf16)(float)lo, a1 = (__bf16)(float)hi;
                w[e] = (uint32_t)__builtin_bit_cast(uint16_t, a0) |
                       ((uint32_t)__builtin_bit_cast(uint16_t, a1) << 16);
            } else {
                w[e] = peak_bf16(peak_hash(seed)) | (peak_bf16(peak_hash(seed + 0x9e3779b9u)) << 16);
            }
        }
        ar[q] = make_uint4(w[0], w[1], w[2], w[3]);
        br[q] = make_uint4(w[4], w[5], w[6], w[7]);
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int t = 0; t < 8; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(pk_bf16x8, ar[t & 3]),
                __builtin_bit_cast(pk_bf16x8, br[(t + (t >> 2)) & 3]), acc[t], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[t][v];
    out[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Second measurement aid: the HBM traffic of one launch of the fused round kernel (per element,
// K error buffers read and written, K replicas read, theta and v read and written) as a flat
// sweep -- one 16-byte position of every array per thread, workgroups in address order, no
// matrix-core work, the same non-temporal accesses.  What it reaches is what the memory system
// gives this mix of streams under the simplest access pattern; the values written are sums of
// what was read and mean nothing.
template <bool TLBF16>
__global__ __launch_bounds__(256) void traffic_probe_kernel(PtrPack<float *> ef,
                                                            PtrPack<const void *> tl, int K,
                                                            float *__restrict__ theta,
                                                            float *__restrict__ vel) {
    typedef float pv4 __attribute__((ext_vector_type(4)));
    typedef uint32_t pu2 __attribute__((ext_vector_type(2)));
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    const pv4 t = __builtin_nontemporal_load(reinterpret_cast<const pv4 *>(theta + i));
    const pv4 v = __builtin_nontemporal_load(reinterpret_cast<const pv4 *>(vel + i));
    pv4 x[DLCX_MAX_WORKERS / 2], l[DLCX_MAX_WORKERS / 2];
    for (int k0 = 0; k0 < K; k0 += DLCX_MAX_WORKERS / 2) {
#pragma unroll
        for (int kk = 0; kk < DLCX_MAX_WORKERS / 2; ++kk) {
            if (k0 + kk < K) {
                x[kk] = __builtin_nontemporal_load(reinterpret_cast<const pv4 *>(ef.p[k0 + kk] + i));
                if (TLBF16) {
                    const pu2 b = __builtin_nontemporal_load(reinterpret_cast<const pu2 *>(
                        reinterpret_cast<const uint16_t *>(tl.p[k0 + kk]) + i));
                    l[kk] = pv4{__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xFFFF0000u),
                                __uint_as_float(b.y << 16), __uint_as_float(b.y & 0xFFFF0000u)};
                } else {
                    l[kk] = __builtin_nontemporal_load(reinterpret_cast<const pv4 *>(
                        reinterpret_cast<const float *>(tl.p[k0 + kk]) + i));
                }
            }
        }
#pragma unroll
        for (int kk = 0; kk < DLCX_MAX_WORKERS / 2; ++kk)
            if (k0 + kk < K)
                __builtin_nontemporal_store((t - l[kk]) + x[kk],
                                            reinterpret_cast<pv4 *>(ef.p[k0 + kk] + i));
    }
    __builtin_nontemporal_store(t + v, reinterpret_cast<pv4 *>(theta + i));
    __builtin_nontemporal_store(t - v, reinterpret_cast<pv4 *>(vel + i));
}

int launch_traffic_probe(int K, const PtrPack<float *> &ef, const PtrPack<const void *> &tl,
                         bool tl_bf16, float *theta, float *vel, int64_t numel, hipStream_t st) {
    Timed timed(KID_TRAFFIC_PROBE, st);
    const dim3 grid((unsigned)(numel / 1024));
    if (tl_bf16)
        hipLaunchKernelGGL(traffic_probe_kernel<true>, grid, dim3(256), 0, st, ef, tl, K, theta, vel);
    else
        hipLaunchKernelGGL(traffic_probe_kernel<false>, grid, dim3(256), 0, st, ef, tl, K, theta, vel);
    return check_launch("traffic_probe");
}

int launch_mfma_peak(int workgroups, int iters, int operands, float *out, hipStream_t st) {
    Timed timed(KID_MFMA_PEAK, st);
    hipLaunchKernelGGL(mfma_peak_kernel, dim3((unsigned)workgroups), dim3(256), 0, st, iters,
                       operands, out);
    return check_launch("mfma_peak");
}

}  // namespace dlcx
