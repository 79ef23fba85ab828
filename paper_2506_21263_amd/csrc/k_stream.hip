// Streaming kernels of the outer step: pseudo-gradient with error compensation (Alg. 2) and the
// Nesterov outer update (Appendix A.3).  Both are pure HBM streams: every thread moves UNROLL
// 16-byte vectors, all loads issued before the first use so that a wave keeps several KB in
// flight.
#include "common.h"

namespace dlcx {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;  // float4 per thread

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}

// Every stream here is touched once per sweep: non-temporal accesses, so that the streams do not
// displace one another in the caches.
typedef float st_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t st_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float4 stream_load4(const float *base, int64_t v) {
    const st_f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const st_f32x4 *>(base) + v);
    return make_float4(x.x, x.y, x.z, x.w);
}
__device__ __forceinline__ uint2 stream_load2(const void *base, int64_t v) {
    const st_u32x2 x = __builtin_nontemporal_load(reinterpret_cast<const st_u32x2 *>(base) + v);
    return make_uint2(x.x, x.y);
}
__device__ __forceinline__ void stream_store4(float *base, int64_t v, const float4 &a) {
    const st_f32x4 x = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(x, reinterpret_cast<st_f32x4 *>(base) + v);
}

template <bool kBf16>
__global__ __launch_bounds__(kThreads) void delta_ef_kernel(const float *__restrict__ theta_g,
                                                            const void *__restrict__ theta_l,
                                                            float *__restrict__ ef,
                                                            int64_t numel) {
    const int64_t nvec = numel >> 2;
    const int64_t base = (int64_t)blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
    float4 g[kUnroll], e[kUnroll], l[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = base + (int64_t)u * kThreads;
        if (v < nvec) {
            g[u] = stream_load4(theta_g, v);
            e[u] = stream_load4(ef, v);
            if (kBf16) {
                const uint2 b = stream_load2(theta_l, v);
                l[u] = make_float4(bf16_bits_to_f32(b.x & 0xFFFFu), bf16_bits_to_f32(b.x >> 16),
                                   bf16_bits_to_f32(b.y & 0xFFFFu), bf16_bits_to_f32(b.y >> 16));
            } else {
                l[u] = stream_load4(reinterpret_cast<const float *>(theta_l), v);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t v = base + (int64_t)u * kThreads;
        if (v < nvec) {
            float4 d;  // summed in fp64, rounded to fp32 once
            d.x = (float)(((double)g[u].x - (double)l[u].x) + (double)e[u].x);
            d.y = (float)(((double)g[u].y - (double)l[u].y) + (double)e[u].y);
            d.z = (float)(((double)g[u].z - (double)l[u].z) + (double)e[u].z);
            d.w = (float)(((double)g[u].w - (double)l[u].w) + (double)e[u].w);
            stream_store4(ef, v, d);
        }
    }
    // ragged tail (numel not a multiple of 4): the last block's first threads
    if (blockIdx.x == gridDim.x - 1) {
        const int64_t x = (nvec << 2) + threadIdx.x;
        if (threadIdx.x < 4 && x < numel) {
            float tl;
            if (kBf16)
                tl = bf16_bits_to_f32(reinterpret_cast<const uint16_t *>(theta_l)[x]);
            else
                tl = reinterpret_cast<const float *>(theta_l)[x];
            ef[x] = (float)(((double)theta_g[x] - (double)tl) + (double)ef[x]);
        }
    }
}

__global__ __launch_bounds__(kThreads) void nesterov_kernel(float *__restrict__ theta,
                                                            float *__restrict__ vel,
                                                            const float *__restrict__ grad,
                                                            int64_t numel, float lr, float mu) {
    const int64_t nvec = numel >> 2;
    const int64_t base = (int64_t)blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
    float4 t[kUnroll], v[kUnroll], g[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t i = base + (int64_t)u * kThreads;
        if (i < nvec) {
            t[u] = stream_load4(theta, i);
            v[u] = stream_load4(vel, i);
            g[u] = stream_load4(grad, i);
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t i = base + (int64_t)u * kThreads;
        if (i < nvec) {
            float4 vn, tn;
            vn.x = fmaf(mu, v[u].x, g[u].x);
            vn.y = fmaf(mu, v[u].y, g[u].y);
            vn.z = fmaf(mu, v[u].z, g[u].z);
            vn.w = fmaf(mu, v[u].w, g[u].w);
            tn.x = fmaf(-lr, fmaf(mu, vn.x, g[u].x), t[u].x);
            tn.y = fmaf(-lr, fmaf(mu, vn.y, g[u].y), t[u].y);
            tn.z = fmaf(-lr, fmaf(mu, vn.z, g[u].z), t[u].z);
            tn.w = fmaf(-lr, fmaf(mu, vn.w, g[u].w), t[u].w);
            stream_store4(vel, i, vn);
            stream_store4(theta, i, tn);
        }
    }
    if (blockIdx.x == gridDim.x - 1) {
        const int64_t x = (nvec << 2) + threadIdx.x;
        if (threadIdx.x < 4 && x < numel) {
            const float vn = fmaf(mu, vel[x], grad[x]);
            theta[x] = fmaf(-lr, fmaf(mu, vn, grad[x]), theta[x]);
            vel[x] = vn;
        }
    }
}

static inline unsigned stream_blocks(int64_t numel) {
    const int64_t per_block = (int64_t)kThreads * kUnroll * 4;
    int64_t b = ceil_div(numel, per_block);
    return (unsigned)(b < 1 ? 1 : b);
}

int launch_delta_ef(const float *theta_g, const void *theta_l, int dtype, float *ef,
                    int64_t numel, hipStream_t st) {
    if (numel == 0) return DLCX_OK;
    const unsigned blocks = stream_blocks(numel);
    Timed timed(KID_DELTA_EF, st);
    if (dtype == DLCX_BF16)
        hipLaunchKernelGGL(delta_ef_kernel<true>, dim3(blocks), dim3(kThreads), 0, st, theta_g,
                           theta_l, ef, numel);
    else
        hipLaunchKernelGGL(delta_ef_kernel<false>, dim3(blocks), dim3(kThreads), 0, st, theta_g,
                           theta_l, ef, numel);
    return check_launch("delta_ef");
}

int launch_nesterov(float *theta, float *v, const float *g, int64_t numel, float lr, float mu,
                    hipStream_t st) {
    if (numel == 0) return DLCX_OK;
    Timed timed(KID_NESTEROV, st);
    hipLaunchKernelGGL(nesterov_kernel, dim3(stream_blocks(numel)), dim3(kThreads), 0, st, theta,
                       v, g, numel, lr, mu);
    return check_launch("outer_nesterov");
}

}  // namespace dlcx
