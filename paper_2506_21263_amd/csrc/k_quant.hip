// QUANTIZE of Alg. 1 (symmetric per-group absmax quantiser, round-half-even) and the
// dequantise-and-average that stands in for the AllReduce of Alg. 2.
//
// One thread owns 4 consecutive elements, so a group of G elements is G/4 adjacent lanes of one
// wavefront and its absmax is a butterfly reduction over those lanes.  Integer decisions are
// taken in fp32 with an IEEE divide, one multiply and v_rndne, exactly as the payload is defined.
#include "common.h"

namespace dlcx {

constexpr int kQThreads = 256;

template <int kLanes>  // lanes per group = group / 4
__device__ __forceinline__ float group_max(float a) {
#pragma unroll
    for (int off = kLanes >> 1; off >= 1; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
    return a;
}

template <int kQbits, int kLanes>
__global__ __launch_bounds__(kQThreads) void quantize_kernel(PtrPack<const float *> xs,
                                                             int64_t nvec,
                                                             PtrPack<uint8_t *> codes,
                                                             PtrPack<float *> scales) {
    const int k = blockIdx.y;
    const float *__restrict__ x = xs.p[k];
    const int64_t v = (int64_t)blockIdx.x * kQThreads + threadIdx.x;
    const bool live = v < nvec;  // whole groups are live or dead together
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) a = reinterpret_cast<const float4 *>(x)[v];
    float amax = fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w)));
    amax = group_max<kLanes>(amax);
    constexpr float qmax = (float)((1 << (kQbits - 1)) - 1);
    float inv = 0.f, scale = 0.f;
    if (amax >= 0x1p-100f) {
        inv = qmax / amax;
        scale = amax / qmax;
    }
    int c0 = (int)fminf(fmaxf(rintf(a.x * inv), -qmax), qmax);
    int c1 = (int)fminf(fmaxf(rintf(a.y * inv), -qmax), qmax);
    int c2 = (int)fminf(fmaxf(rintf(a.z * inv), -qmax), qmax);
    int c3 = (int)fminf(fmaxf(rintf(a.w * inv), -qmax), qmax);
    if (!live) return;
    if (kQbits == 4) {
        const uint32_t packed = (uint32_t)(c0 & 0xF) | ((uint32_t)(c1 & 0xF) << 4) |
                                ((uint32_t)(c2 & 0xF) << 8) | ((uint32_t)(c3 & 0xF) << 12);
        reinterpret_cast<uint16_t *>(codes.p[k])[v] = (uint16_t)packed;
    } else {
        const uint32_t packed = (uint32_t)(c0 & 0xFF) | ((uint32_t)(c1 & 0xFF) << 8) |
                                ((uint32_t)(c2 & 0xFF) << 16) | ((uint32_t)(c3 & 0xFF) << 24);
        reinterpret_cast<uint32_t *>(codes.p[k])[v] = packed;
    }
    if ((threadIdx.x & (kLanes - 1)) == 0) scales.p[k][v / kLanes] = scale;
}

// Mean of K decoded payloads: fp64 sum of the (exact) products code * scale in worker order, one
// rounding to fp32 at the end.
template <int kQbits>
__global__ __launch_bounds__(kQThreads) void dequant_average_kernel(
    int K, PtrPack<const uint8_t *> codes, PtrPack<const float *> scales, int64_t nvec,
    int lanes_per_group, double inv_k, int exact_inv, float *__restrict__ out) {
    const int64_t v = (int64_t)blockIdx.x * kQThreads + threadIdx.x;
    if (v >= nvec) return;
    const int64_t g = v / lanes_per_group;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    for (int k = 0; k < K; ++k) {  // workers in index order
        const double s = (double)scales.p[k][g];
        int c0, c1, c2, c3;
        if (kQbits == 4) {
            const uint32_t w = reinterpret_cast<const uint16_t *>(codes.p[k])[v];
            c0 = ((int)(w << 28)) >> 28;
            c1 = ((int)(w << 24)) >> 28;
            c2 = ((int)(w << 20)) >> 28;
            c3 = ((int)(w << 16)) >> 28;
        } else {
            const uint32_t w = reinterpret_cast<const uint32_t *>(codes.p[k])[v];
            c0 = ((int)(w << 24)) >> 24;
            c1 = ((int)(w << 16)) >> 24;
            c2 = ((int)(w << 8)) >> 24;
            c3 = ((int)w) >> 24;
        }
        a0 = fma((double)c0, s, a0);
        a1 = fma((double)c1, s, a1);
        a2 = fma((double)c2, s, a2);
        a3 = fma((double)c3, s, a3);
    }
    if (exact_inv) {  // K a power of two: the reciprocal and the product are exact
        a0 *= inv_k; a1 *= inv_k; a2 *= inv_k; a3 *= inv_k;
    } else {
        const double kd = (double)K;
        a0 /= kd; a1 /= kd; a2 /= kd; a3 /= kd;
    }
    reinterpret_cast<float4 *>(out)[v] = make_float4((float)a0, (float)a1, (float)a2, (float)a3);
}

template <int kQbits>
static int quantize_dispatch(int K, const PtrPack<const float *> &x, int64_t nvec, int group,
                             const PtrPack<uint8_t *> &codes, const PtrPack<float *> &scales,
                             hipStream_t st) {
    const dim3 grid((unsigned)ceil_div(nvec, kQThreads), (unsigned)K);
    const dim3 block(kQThreads);
    Timed timed(KID_QUANTIZE, st);
    switch (group) {
        case 16: hipLaunchKernelGGL((quantize_kernel<kQbits, 4>), grid, block, 0, st, x, nvec, codes, scales); break;
        case 32: hipLaunchKernelGGL((quantize_kernel<kQbits, 8>), grid, block, 0, st, x, nvec, codes, scales); break;
        case 64: hipLaunchKernelGGL((quantize_kernel<kQbits, 16>), grid, block, 0, st, x, nvec, codes, scales); break;
        case 128: hipLaunchKernelGGL((quantize_kernel<kQbits, 32>), grid, block, 0, st, x, nvec, codes, scales); break;
        case 256: hipLaunchKernelGGL((quantize_kernel<kQbits, 64>), grid, block, 0, st, x, nvec, codes, scales); break;
        default: return DLCX_EINVAL;
    }
    return check_launch("quantize");
}

int launch_quantize(int K, const PtrPack<const float *> &x, int64_t count, int qbits, int group,
                    const PtrPack<uint8_t *> &codes, const PtrPack<float *> &scales,
                    hipStream_t st) {
    if (count == 0 || K == 0) return DLCX_OK;
    const int64_t nvec = count >> 2;
    if (qbits == 4) return quantize_dispatch<4>(K, x, nvec, group, codes, scales, st);
    return quantize_dispatch<8>(K, x, nvec, group, codes, scales, st);
}

int launch_dequant_average(int K, const PtrPack<const uint8_t *> &codes,
                           const PtrPack<const float *> &scales, int64_t count, int qbits,
                           int group, float *mean_out, hipStream_t st) {
    if (count == 0) return DLCX_OK;
    const int64_t nvec = count >> 2;
    const dim3 grid((unsigned)ceil_div(nvec, kQThreads));
    const double inv_k = 1.0 / (double)K;
    const int exact_inv = (K & (K - 1)) == 0;
    Timed timed(KID_DEQUANT_AVG, st);
    if (qbits == 4)
        hipLaunchKernelGGL(dequant_average_kernel<4>, grid, dim3(kQThreads), 0, st, K, codes,
                           scales, nvec, group / 4, inv_k, exact_inv, mean_out);
    else
        hipLaunchKernelGGL(dequant_average_kernel<8>, grid, dim3(kQThreads), 0, st, K, codes,
                           scales, nvec, group / 4, inv_k, exact_inv, mean_out);
    return check_launch("dequant_average");
}

}  // namespace dlcx
