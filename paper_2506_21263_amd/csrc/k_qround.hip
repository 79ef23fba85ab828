// Outer step of Alg. 2 for a tensor whose compressor is the quantiser alone (Alg. 1 without the
// LOWRANK step: the Int4-only setting of Sec. 4.1, and the only form that applies to tensors
// that are not matrices).  Everything between two quantisations happens in one sweep:
//
//   d        = mean_k dequant(previous payload_k)          (re-encoded to q bits if requested)
//   e_k      = delta_k - d ;  delta_k = (theta - theta_l,k) + e_k      -> stored over delta_k
//   payload_k = QUANTIZE(delta_k)                           (codes + one fp32 scale per group)
//   v <- mu v + d ;  theta <- theta - lr (d + mu v)         (OuterOpt, one step late; in fp64)
//
// The averaged pseudo-gradient is never written: the K payloads are the only form in which it
// exists between two outer steps, which is also what would travel between workers.
//
// One thread owns 4 consecutive elements; a group of G elements is G/4 adjacent lanes of one
// wavefront.  The mean is accumulated in fp64 in worker order and rounded to fp32 once, and so is
// the sum (theta - theta_l) + e; every other operation is the fp32 operation of the definition.
// No result depends on the launch shape.
#include "common.h"

// every product and sum below is a rounding of the definition: no fused multiply-add unless written
#pragma clang fp contract(off)

namespace dlcx {

constexpr int kQrThreads = 256;

// 16-byte accesses of data that is touched once per outer step: marked non-temporal so that they
// do not displace one another in the caches
typedef float qr_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load4(const float *p) {
    const qr_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const qr_f32x4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store4(float *p, const float4 &a) {
    const qr_f32x4 v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<qr_f32x4 *>(p));
}

template <int kLanes>
__device__ __forceinline__ float qr_group_max(float a) {
#pragma unroll
    for (int off = kLanes >> 1; off >= 1; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
    return a;
}

// QUANTIZE of Alg. 1 for this lane's 4 elements of a group spread over kLanes lanes
template <int kQbits, int kLanes>
__device__ __forceinline__ void quantize4(const float4 &a, int (&c)[4], float &scale) {
    float amax = fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w)));
    amax = qr_group_max<kLanes>(amax);
    constexpr float qmax = (float)((1 << (kQbits - 1)) - 1);
    float inv = 0.f;
    scale = 0.f;
    if (amax >= 0x1p-100f) {
        inv = qmax / amax;
        scale = amax / qmax;
    }
    c[0] = (int)fminf(fmaxf(rintf(a.x * inv), -qmax), qmax);
    c[1] = (int)fminf(fmaxf(rintf(a.y * inv), -qmax), qmax);
    c[2] = (int)fminf(fmaxf(rintf(a.z * inv), -qmax), qmax);
    c[3] = (int)fminf(fmaxf(rintf(a.w * inv), -qmax), qmax);
}

template <int kQbits>
__device__ __forceinline__ void load_codes4(const uint8_t *codes, int64_t v, int (&c)[4]) {
    if (kQbits == 4) {
        const uint32_t w = reinterpret_cast<const uint16_t *>(codes)[v];
        c[0] = ((int)(w << 28)) >> 28;
        c[1] = ((int)(w << 24)) >> 28;
        c[2] = ((int)(w << 20)) >> 28;
        c[3] = ((int)(w << 16)) >> 28;
    } else {
        const uint32_t w = reinterpret_cast<const uint32_t *>(codes)[v];
        c[0] = ((int)(w << 24)) >> 24;
        c[1] = ((int)(w << 16)) >> 24;
        c[2] = ((int)(w << 8)) >> 24;
        c[3] = ((int)w) >> 24;
    }
}

template <int kQbits>
__device__ __forceinline__ void store_codes4(uint8_t *codes, int64_t v, const int (&c)[4]) {
    if (kQbits == 4) {
        const uint32_t packed = (uint32_t)(c[0] & 0xF) | ((uint32_t)(c[1] & 0xF) << 4) |
                                ((uint32_t)(c[2] & 0xF) << 8) | ((uint32_t)(c[3] & 0xF) << 12);
        reinterpret_cast<uint16_t *>(codes)[v] = (uint16_t)packed;
    } else {
        const uint32_t packed = (uint32_t)(c[0] & 0xFF) | ((uint32_t)(c[1] & 0xFF) << 8) |
                                ((uint32_t)(c[2] & 0xFF) << 16) | ((uint32_t)(c[3] & 0xFF) << 24);
        reinterpret_cast<uint32_t *>(codes)[v] = packed;
    }
}

// mean of K decoded payloads for this lane's 4 elements: fp64 sum in worker order, one rounding
template <int kQbits>
__device__ __forceinline__ float4 mean4(int K, const PtrPack<const uint8_t *> &codes,
                                        const PtrPack<const float *> &scales, int64_t v, int64_t g,
                                        double inv_k, bool exact_inv) {
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    for (int k = 0; k < K; ++k) {
        const double s = (double)scales.p[k][g];
        int c[4];
        load_codes4<kQbits>(codes.p[k], v, c);
        a0 = fma((double)c[0], s, a0);  // the product is exact in fp64
        a1 = fma((double)c[1], s, a1);
        a2 = fma((double)c[2], s, a2);
        a3 = fma((double)c[3], s, a3);
    }
    if (exact_inv) {  // K a power of two: the reciprocal is exact and so is the product
        a0 *= inv_k; a1 *= inv_k; a2 *= inv_k; a3 *= inv_k;
    } else {
        const double kd = (double)K;
        a0 /= kd; a1 /= kd; a2 /= kd; a3 /= kd;
    }
    return make_float4((float)a0, (float)a1, (float)a2, (float)a3);
}

struct QRoundArgs {
    int K;
    int has_prev;  // 0 at the first outer step: nothing to feed back and nothing to apply
    int64_t nvec;  // numel / 4
    PtrPack<const void *> tl;
    PtrPack<float *> ef;
    float *theta, *vel;
    double lr, mu;
    double inv_k;
    int exact_inv;
    PtrPack<const uint8_t *> pcodes;
    PtrPack<const float *> pscales;
    PtrPack<uint8_t *> codes;
    PtrPack<float *> scales;
};

template <int kQbits, int kLanes, bool kBf16, bool kRequant>
__global__ __launch_bounds__(kQrThreads) void quant_round_kernel(QRoundArgs a) {
    const int64_t v = (int64_t)blockIdx.x * kQrThreads + threadIdx.x;
    const bool live = v < a.nvec;  // whole groups are live or dead together
    // a dead lane reads vector 0 instead of skipping its loads behind a per-lane condition (the
    // loop of loads then is one block that the compiler can issue together); it stores nothing
    const int64_t vc = live ? v : 0;
    const int64_t g = vc / kLanes;
    float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
    if (a.has_prev) {
        d = mean4<kQbits>(a.K, a.pcodes, a.pscales, vc, g, a.inv_k, a.exact_inv != 0);
        if (kRequant) {  // the mean as a q-bit reduction would hand it on
            int c[4];
            float s;
            quantize4<kQbits, kLanes>(d, c, s);
            d = make_float4((float)c[0] * s, (float)c[1] * s, (float)c[2] * s, (float)c[3] * s);
        }
    }
    float4 t = stream_load4(a.theta + 4 * vc), vel = make_float4(0.f, 0.f, 0.f, 0.f);
    if (a.has_prev) vel = stream_load4(a.vel + 4 * vc);
    for (int k = 0; k < a.K; ++k) {
        float4 x = stream_load4(a.ef.p[k] + 4 * vc), l;
        if (kBf16) {
            const uint2 b = reinterpret_cast<const uint2 *>(a.tl.p[k])[vc];
            l = make_float4(__uint_as_float(b.x << 16), __uint_as_float(b.x & 0xFFFF0000u),
                            __uint_as_float(b.y << 16), __uint_as_float(b.y & 0xFFFF0000u));
        } else {
            l = reinterpret_cast<const float4 *>(a.tl.p[k])[vc];
        }
        if (a.has_prev) {  // e = delta - d of the previous step (one fp32 rounding)
            x.x -= d.x;
            x.y -= d.y;
            x.z -= d.z;
            x.w -= d.w;
        }
        // the new pseudo-gradient (theta - theta_l) + e: summed in fp64, rounded to fp32 once
        float4 dl;
        dl.x = (float)(((double)t.x - (double)l.x) + (double)x.x);
        dl.y = (float)(((double)t.y - (double)l.y) + (double)x.y);
        dl.z = (float)(((double)t.z - (double)l.z) + (double)x.z);
        dl.w = (float)(((double)t.w - (double)l.w) + (double)x.w);
        int c[4];
        float s;
        quantize4<kQbits, kLanes>(dl, c, s);
        if (live) {
            stream_store4(a.ef.p[k] + 4 * vc, dl);
            store_codes4<kQbits>(a.codes.p[k], vc, c);
            if ((threadIdx.x & (kLanes - 1)) == 0) a.scales.p[k][g] = s;
        }
    }
    if (a.has_prev && live) {  // OuterOpt in fp64, each result rounded to fp32 once
        const float dd[4] = {d.x, d.y, d.z, d.w};
        const float vo[4] = {vel.x, vel.y, vel.z, vel.w};
        const float to[4] = {t.x, t.y, t.z, t.w};
        float vn[4], tn[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const double vd = a.mu * (double)vo[q] + (double)dd[q];
            const double td = (double)to[q] - a.lr * ((double)dd[q] + a.mu * vd);
            vn[q] = (float)vd;
            tn[q] = (float)td;
        }
        stream_store4(a.vel + 4 * vc, make_float4(vn[0], vn[1], vn[2], vn[3]));
        stream_store4(a.theta + 4 * vc, make_float4(tn[0], tn[1], tn[2], tn[3]));
    }
}

template <int kQbits, int kLanes>
static void quant_round_launch(const QRoundArgs &a, bool bf16, bool requant, hipStream_t st) {
    const dim3 grid((unsigned)ceil_div(a.nvec, kQrThreads)), block(kQrThreads);
    if (bf16) {
        if (requant)
            hipLaunchKernelGGL((quant_round_kernel<kQbits, kLanes, true, true>), grid, block, 0, st, a);
        else
            hipLaunchKernelGGL((quant_round_kernel<kQbits, kLanes, true, false>), grid, block, 0, st, a);
    } else {
        if (requant)
            hipLaunchKernelGGL((quant_round_kernel<kQbits, kLanes, false, true>), grid, block, 0, st, a);
        else
            hipLaunchKernelGGL((quant_round_kernel<kQbits, kLanes, false, false>), grid, block, 0, st, a);
    }
}

template <int kQbits>
static int quant_round_dispatch(const QRoundArgs &a, int group, bool bf16, bool requant,
                                hipStream_t st) {
    switch (group) {
        case 16: quant_round_launch<kQbits, 4>(a, bf16, requant, st); break;
        case 32: quant_round_launch<kQbits, 8>(a, bf16, requant, st); break;
        case 64: quant_round_launch<kQbits, 16>(a, bf16, requant, st); break;
        case 128: quant_round_launch<kQbits, 32>(a, bf16, requant, st); break;
        case 256: quant_round_launch<kQbits, 64>(a, bf16, requant, st); break;
        default: return DLCX_EINVAL;
    }
    return check_launch("quant_round");
}

int launch_quant_round(int64_t numel, int qbits, int group, int K, const PtrPack<const void *> &tl,
                       int tl_dtype, const PtrPack<float *> &ef, float *theta, float *vel, double lr,
                       double mu, bool has_prev, const PtrPack<const uint8_t *> &pcodes,
                       const PtrPack<const float *> &pscales, bool requant,
                       const PtrPack<uint8_t *> &codes, const PtrPack<float *> &scales,
                       hipStream_t st) {
    if (numel == 0) return DLCX_OK;
    QRoundArgs a;
    a.K = K;
    a.has_prev = has_prev ? 1 : 0;
    a.nvec = numel >> 2;
    a.tl = tl;
    a.ef = ef;
    a.theta = theta;
    a.vel = vel;
    a.lr = lr;
    a.mu = mu;
    a.inv_k = 1.0 / (double)K;
    a.exact_inv = (K & (K - 1)) == 0;
    a.pcodes = pcodes;
    a.pscales = pscales;
    a.codes = codes;
    a.scales = scales;
    Timed timed(KID_QUANT_ROUND, st);
    if (qbits == 4) return quant_round_dispatch<4>(a, group, tl_dtype == DLCX_BF16, requant, st);
    return quant_round_dispatch<8>(a, group, tl_dtype == DLCX_BF16, requant, st);
}

// ---------------------------------------------------------------------------------------------
// x <- dequant(QUANTIZE(x)) in place: a mean re-encoded to q bits.
// ---------------------------------------------------------------------------------------------
template <int kQbits, int kLanes>
__global__ __launch_bounds__(kQrThreads) void requantize_kernel(float *__restrict__ x,
                                                                int64_t nvec) {
    const int64_t v = (int64_t)blockIdx.x * kQrThreads + threadIdx.x;
    const bool live = v < nvec;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    if (live) a = reinterpret_cast<const float4 *>(x)[v];
    int c[4];
    float s;
    quantize4<kQbits, kLanes>(a, c, s);
    if (live)
        reinterpret_cast<float4 *>(x)[v] =
            make_float4((float)c[0] * s, (float)c[1] * s, (float)c[2] * s, (float)c[3] * s);
}

template <int kQbits>
static int requantize_dispatch(float *x, int64_t nvec, int group, hipStream_t st) {
    const dim3 grid((unsigned)ceil_div(nvec, kQrThreads)), block(kQrThreads);
    switch (group) {
        case 16: hipLaunchKernelGGL((requantize_kernel<kQbits, 4>), grid, block, 0, st, x, nvec); break;
        case 32: hipLaunchKernelGGL((requantize_kernel<kQbits, 8>), grid, block, 0, st, x, nvec); break;
        case 64: hipLaunchKernelGGL((requantize_kernel<kQbits, 16>), grid, block, 0, st, x, nvec); break;
        case 128: hipLaunchKernelGGL((requantize_kernel<kQbits, 32>), grid, block, 0, st, x, nvec); break;
        case 256: hipLaunchKernelGGL((requantize_kernel<kQbits, 64>), grid, block, 0, st, x, nvec); break;
        default: return DLCX_EINVAL;
    }
    return check_launch("requantize");
}

int launch_requantize(float *x, int64_t count, int qbits, int group, hipStream_t st) {
    if (count == 0) return DLCX_OK;
    Timed timed(KID_REQUANT, st);
    if (qbits == 4) return requantize_dispatch<4>(x, count >> 2, group, st);
    return requantize_dispatch<8>(x, count >> 2, group, st);
}

// ---------------------------------------------------------------------------------------------
// Error buffers of Alg. 2 for K workers against a materialised average:  e_k <- delta_k - d.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kQrThreads) void ef_update_kernel(int K, PtrPack<float *> ef,
                                                               const float *__restrict__ d,
                                                               int64_t numel) {
    const int64_t nvec = numel >> 2;
    const int64_t v = (int64_t)blockIdx.x * kQrThreads + threadIdx.x;
    if (v < nvec) {
        const float4 dd = reinterpret_cast<const float4 *>(d)[v];
        for (int k = 0; k < K; ++k) {
            float4 e = reinterpret_cast<const float4 *>(ef.p[k])[v];
            e.x -= dd.x;
            e.y -= dd.y;
            e.z -= dd.z;
            e.w -= dd.w;
            reinterpret_cast<float4 *>(ef.p[k])[v] = e;
        }
    }
    if (blockIdx.x == gridDim.x - 1) {  // ragged tail
        const int64_t x = (nvec << 2) + threadIdx.x;
        if (threadIdx.x < 4 && x < numel)
            for (int k = 0; k < K; ++k) ef.p[k][x] -= d[x];
    }
}

int launch_ef_update(int K, const PtrPack<float *> &ef, const float *d, int64_t numel,
                     hipStream_t st) {
    if (numel == 0 || K == 0) return DLCX_OK;
    int64_t blocks = ceil_div(numel >> 2, kQrThreads);
    if (blocks < 1) blocks = 1;
    Timed timed(KID_EF_UPDATE, st);
    hipLaunchKernelGGL(ef_update_kernel, dim3((unsigned)blocks), dim3(kQrThreads), 0, st, K, ef, d,
                       numel);
    return check_launch("ef_update");
}

}  // namespace dlcx
