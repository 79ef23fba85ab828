// Rank-r products of the low-rank compressor on the bf16 matrix cores of gfx950
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation).
//
// Every fp32 operand is split into NS bf16 pieces, x = x0 + x1 (+ x2), each piece the bf16
// rounding of what the earlier pieces left over, and a product a*b is the sum of the piece
// products whose weight is not below the last piece:
//     NS = 2 (DLCX_MMA_BF16):  a0b0 + a0b1 + a1b0               error ~ 2^-17 per product
//     NS = 3 (DLCX_MMA_F32):   + a1b1 + a0b2 + a2b0             error ~ 2^-24 per product
// so the matrix cores run 3 or 6 bf16 instructions per 32x32x16 block.  At the ranks of interest
// the products are bound by the HBM stream of delta (4 bytes per element against 6r or 12r
// flops), not by the matrix cores, which is why the extra instructions are affordable; the native
// fp32 MFMA would cost 16 instruction issues of twice the latency for the same block.
//
// Operand layout of v_mfma_f32_32x32x16_bf16 (D = A B + C, A is 32 x 16, B is 16 x 32):
//   lane l holds A[l % 32][8 (l / 32) + e] and B[8 (l / 32) + e][l % 32], e = 0..7 (16 bytes);
//   D[i][j] is in lane j + 32 ((i / 4) % 2), register (i % 4) + 4 (i / 8).
// The small operand of every product (the basis, or both factors of the reconstruction) is first
// repacked ("fragments") so that a wavefront fetches one 32 x 16 operand block of one piece as
// 1 KB of consecutive memory; fragments are read straight from L2 into registers.  The big
// operand delta is staged through LDS (P phase, reduction along a row) or loaded straight into
// the operand layout with 128-byte row segments (Q phase, reduction down a column).
//
// Kernels in this file:
//   pack_kcontig_kernel / pack_kstrided_kernel   fragments of a basis / of a factor
//   project_p_mfma_kernel, project_q_mfma_kernel  projections, every wavefront does everything
//                                                 (r <= 32, and P for matrices with few rows)
//   project_p_ws_kernel, project_q_ws_kernel      projections with producer and consumer
//                                                 wavefronts (r > 32)
//   reconstruct_mfma_kernel                       Delta_hat tile by tile with the elementwise
//                                                 steps of Alg. 2 fused in (any rank)
//   round_mfma_kernel                             the same plus the P phase of the next
//                                                 compression: the benchmark's hot kernel (r <= 64)
// Two things learnt on this hardware shape all of them.  A wavefront's loads return in order, so
// a wait for something needed soon (a fragment from L2) also waits for everything requested
// before it (delta from HBM, needed much later): requests are issued in the order of need, or
// the two kinds of load are given to different wavefronts.  And a load behind a per-lane
// condition cuts the loop into small blocks that the compiler schedules one by one: lanes
// outside the matrix read a valid address instead and the value is dropped.
#include <type_traits>

#include "common.h"

namespace dlcx {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kW = 256;  // threads per workgroup (4 wavefronts)

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {  // round-to-nearest-even
    const f32x2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ uint32_t pack_f16x2(float a, float b) {  // round-to-nearest-even
    typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2_t));
}

// pieces of the pair (a, b): out[h] holds piece h of a in its low half, of b in its high half.
// NS == 1 is the fp16 form of an operand: one piece, the fp16 rounding of the value (the caller
// has scaled it into fp16's range by a power of two).
template <int NS>
__device__ __forceinline__ void split2(float a, float b, uint32_t (&out)[NS]) {
    if constexpr (NS == 1) {
        out[0] = pack_f16x2(a, b);
        return;
    }
#pragma unroll
    for (int h = 0; h < NS; ++h) {
        const uint32_t p = pack_bf16x2(a, b);
        out[h] = p;
        if (h + 1 < NS) {
            a -= __uint_as_float(p << 16);
            b -= __uint_as_float(p & 0xFFFF0000u);
        }
    }
}

// 8 consecutive-k values -> NS operand registers (uint4 = 8 bf16)
template <int NS>
__device__ __forceinline__ void split8(const float (&x)[8], uint4 (&out)[NS]) {
    uint32_t p[4][NS];
#pragma unroll
    for (int q = 0; q < 4; ++q) split2<NS>(x[2 * q], x[2 * q + 1], p[q]);
#pragma unroll
    for (int h = 0; h < NS; ++h) out[h] = make_uint4(p[0][h], p[1][h], p[2][h], p[3][h]);
}

__device__ __forceinline__ f32x16_t mfma(const uint4 &a, const uint4 &b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

template <int NS>
__device__ __forceinline__ void mfma_split(const uint4 (&a)[NS], const uint4 (&b)[NS],
                                           f32x16_t &c) {
    if constexpr (NS == 1) {  // one fp16 product
        typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
        c = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a[0]),
                                                   __builtin_bit_cast(f16x8_t, b[0]), c, 0, 0, 0);
        return;
    }
    if (NS == 3) {  // smallest terms first
        c = mfma(a[2], b[0], c);
        c = mfma(a[0], b[2], c);
        c = mfma(a[1], b[1], c);
    }
    if (NS >= 2) {
        c = mfma(a[1], b[0], c);
        c = mfma(a[0], b[1], c);
    }
    c = mfma(a[0], b[0], c);
}

// row of D held in register v of lane `lane`
__device__ __forceinline__ int d_row(int v, int lane) {
    return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
}

// Accesses to the big streams (delta, theta_l, theta, v), each touched once per sweep: marked
// non-temporal so that they do not displace the fragments and one another in the caches.
typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t nt_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float4 stream_load4(const float *p) {
    const nt_f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 stream_load2(const void *p) {
    const nt_u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const nt_u32x2 *>(p));
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ void stream_store4(float *p, const float4 &a) {
    const nt_f32x4 v = {a.x, a.y, a.z, a.w};
    __builtin_nontemporal_store(v, reinterpret_cast<nt_f32x4 *>(p));
}

// ---------------------------------------------------------------------------------------------
// Fragment packing.
// ---------------------------------------------------------------------------------------------
// src is nrows x L with the reduction index contiguous (a basis: Q_in is r x n, P_hat is r x m).
// Fragment (s, rb, h): rows rb*32 .. +32, reduction indices s*16 .. +16, piece h, at
// frags[((s * RB + rb) * NS + h) * 64 + lane].  Rows >= nrows and indices >= L are zero.
template <int NS>
__global__ __launch_bounds__(kW) void pack_kcontig_kernel(const float *__restrict__ src,
                                                          int nrows, int64_t L, int RB,
                                                          int64_t KS, uint4 *__restrict__ frags,
                                                          const float *__restrict__ row_scale) {
    const int64_t f = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (f >= KS * RB) return;
    const int64_t s = f / RB;
    const int rb = (int)(f % RB);
    const int row = rb * 32 + (lane & 31);
    const int64_t k0 = s * 16 + (lane >> 5) * 8;
    float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (row < nrows && k0 < L) {  // L is a multiple of 8
        const float4 a = *reinterpret_cast<const float4 *>(src + (int64_t)row * L + k0);
        const float4 b = *reinterpret_cast<const float4 *>(src + (int64_t)row * L + k0 + 4);
        x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
        x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
        if (row_scale) {  // a power of two per row: exact
            const float sc = row_scale[row];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] *= sc;
        }
    }
    uint4 out[NS];
    split8<NS>(x, out);
#pragma unroll
    for (int h = 0; h < NS; ++h) frags[(f * NS + h) * 64 + lane] = out[h];
}

// The fp16 form of a projection (NS == 1) needs its operands inside fp16's range.  delta is
// multiplied by 2^kF16DeltaShift, which is safe while the largest |delta| of the launch lies in
// [2^-14, 15.99) (the kernel records it; outside that window the bf16 kernel redoes the launch).
// Every row of the basis (one factor column) gets its own power of two that puts its largest
// entry into [2^7, 2^8): in_scale[c] for the fragments, out_scale[c] = 2^-kF16DeltaShift /
// in_scale[c] for the result, so that scaling is exact and invisible.  Workgroup c handles row c;
// workgroup 0 also clears the launch's record of the largest |delta|.
constexpr int kF16DeltaShift = 12;
__global__ __launch_bounds__(kW) void basis_scale_kernel(const float *__restrict__ src, int64_t L,
                                                         float *__restrict__ in_scale,
                                                         float *__restrict__ out_scale,
                                                         uint32_t *__restrict__ amax_record) {
    __shared__ float red[kW];
    const int c = blockIdx.x;
    float a = 0.f;
    for (int64_t i = threadIdx.x * 4; i < L; i += kW * 4) {  // L is a multiple of 8
        const float4 v = *reinterpret_cast<const float4 *>(src + (int64_t)c * L + i);
        a = fmaxf(fmaxf(a, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
    red[threadIdx.x] = a;
    __syncthreads();
    for (int s = kW / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float amax = red[0];
        int e = 0;
        if (amax > 0.f && amax < 3.0e38f) e = 7 - ilogbf(amax);
        e = e < -100 ? -100 : (e > 100 ? 100 : e);
        in_scale[c] = ldexpf(1.f, e);
        out_scale[c] = ldexpf(1.f, -e - kF16DeltaShift);
        if (c == 0) *amax_record = 0u;
    }
}

// Did the fp16 form of the launch see its operands in range?  (largest |delta| as fp32 bits)
__device__ __forceinline__ bool f16_range_ok(uint32_t amax_bits) {
    const float a = __uint_as_float(amax_bits);
    return a >= 0x1p-14f && a < 15.99f;
}

// largest |x| over a wavefront, then one atomic per wavefront (bit patterns of non-negative
// floats order like the floats)
__device__ __forceinline__ void record_amax(float a, uint32_t *record) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off, 64));
    if ((threadIdx.x & 63) == 0) atomicMax(record, __float_as_uint(a));
}

// src is r x L with the reduction index c strided (a factor used in the reconstruction).
// Fragment (xb, s, h): positions xb*32 .. +32 along L, reduction indices s*16 .. +16, at
// frags[((xb * KS + s) * NS + h) * 64 + lane].
template <int NS>
__global__ __launch_bounds__(kW) void pack_kstrided_kernel(const float *__restrict__ src, int r,
                                                           int64_t L, int KS, int64_t XB,
                                                           uint4 *__restrict__ frags) {
    const int64_t f = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (f >= XB * KS) return;
    const int64_t xb = f / KS;
    const int s = (int)(f % KS);
    const int64_t x0 = xb * 32 + (lane & 31);
    const int c0 = s * 16 + (lane >> 5) * 8;
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
        x[e] = (x0 < L && c0 + e < r) ? src[(int64_t)(c0 + e) * L + x0] : 0.f;
    uint4 out[NS];
    split8<NS>(x, out);
#pragma unroll
    for (int h = 0; h < NS; ++h) frags[(f * NS + h) * 64 + lane] = out[h];
}

// ---------------------------------------------------------------------------------------------
// P phase:  P_k[i][c] = sum_j delta_k[i][j] Q_in[c][j].
// Workgroup: RB row blocks (32 RB rows) of delta, swept along j in stages of 64 (4 k-steps).
// The 4 wavefronts split the work as WC (groups of CBW basis blocks) x WK (halves of a stage) x
// WR (groups of row blocks).  A = basis fragments (M = c), B = delta from LDS (N = i): D[c][i].
// A basis fragment serves RB / WR row blocks once it is in registers, so the fragment traffic
// per byte of delta falls with RB: at r = 256 it is 4 : 1 with 64 rows and 2 : 1 with 128, which
// is what lets the matrix cores, not L2, set the pace there.
// ---------------------------------------------------------------------------------------------
constexpr int kPPitch = 64 * 2 + 16;  // bytes per LDS row of one piece: 64 bf16 + pad

// Workgroup barrier for data exchanged through LDS: every LDS access of this wavefront has
// completed before it arrives, and the compiler moves no memory access across.  Global loads
// that are still outstanding (the next stage, already requested) are NOT waited for, which
// __syncthreads() would do.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int NS, int CBW, int WC, int WK, int WR, int RB>
constexpr int project_p_lds_bytes() {
    constexpr int buf = 2 * NS * 32 * RB * kPPitch;
    constexpr int red = (WK == 2) ? 2 * CBW * (RB / WR) * 16 * 64 * 4 : 0;
    return buf > red ? buf : red;
}

template <int NS, int CBW, int WC, int WK, int WR, int RB>
__global__ __launch_bounds__(kW) void project_p_mfma_kernel(PtrPack<const float *> deltas,
                                                            const uint4 *__restrict__ afrags,
                                                            PtrPack<float *> outs, int64_t m,
                                                            int64_t n, int r) {
    constexpr int CB = CBW * WC;
    constexpr int RBW = RB / WR;
    constexpr int KSW = 4 / WK;
    constexpr int kRows = 32 * RB;
    constexpr int kVec = kRows * 16 / kW;  // float4 per thread and stage
    static_assert(WC * WK * WR == 4, "four wavefronts");
    constexpr int kBuf = NS * kRows * kPPitch;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const float *__restrict__ delta = deltas.p[blockIdx.y];
    float *__restrict__ out = outs.p[blockIdx.y];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wc = wave % WC, wk = (wave / WC) % WK, wr = wave / (WC * WK);
    const int64_t i0 = (int64_t)blockIdx.x * kRows;
    const int64_t nstages = (n + 63) / 64;

    f32x16_t acc[CBW][RBW];
#pragma unroll
    for (int a = 0; a < CBW; ++a)
#pragma unroll
        for (int b = 0; b < RBW; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    // this thread's float4 of a stage: (row, 4 columns)
    float4 pre[kVec];
    auto load_stage = [&](int64_t t) {
#pragma unroll
        for (int u = 0; u < kVec; ++u) {
            const int idx = tid + kW * u;
            const int row = idx >> 4, c4 = idx & 15;
            const int64_t j = t * 64 + c4 * 4;
            pre[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + row < m && j < n)
                pre[u] = stream_load4(delta + (i0 + row) * n + j);
        }
    };
    // basis fragments of a stage: fetched one stage ahead, so that the matrix cores do not wait
    // for L2 after every barrier -- except in the 4-block shape, where the second copy of the
    // fragments costs a wavefront per SIMD and the kernel comes out slower
    constexpr bool kAhead = !(CBW == 2 && WC == 2);
    uint4 a[KSW][CBW][NS];
    auto load_frags = [&](uint4 (&dst)[KSW][CBW][NS], int64_t t) {
#pragma unroll
        for (int ks = 0; ks < KSW; ++ks)
#pragma unroll
            for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
                for (int h = 0; h < NS; ++h) {
                    const int64_t sg = t * 4 + wk * KSW + ks;
                    dst[ks][cb][h] = afrags[((sg * CB + wc * CBW + cb) * NS + h) * 64 + lane];
                }
    };
    if (kAhead && nstages > 0) load_frags(a, 0);
    load_stage(0);
    for (int64_t t = 0; t < nstages; ++t) {
        unsigned char *buf = lds + (t & 1) * kBuf;
#pragma unroll
        for (int u = 0; u < kVec; ++u) {
            const int idx = tid + kW * u;
            const int row = idx >> 4, c4 = idx & 15;
            uint32_t lo[NS], hi[NS];
            split2<NS>(pre[u].x, pre[u].y, lo);
            split2<NS>(pre[u].z, pre[u].w, hi);
#pragma unroll
            for (int h = 0; h < NS; ++h)
                *reinterpret_cast<uint2 *>(buf + (h * kRows + row) * kPPitch + c4 * 8) =
                    make_uint2(lo[h], hi[h]);
        }
        // the next stage's fragments are requested before the next stage of delta, so that
        // waiting for them later does not wait for that stage as well
        uint4 an[KSW][CBW][NS];  // unused (and removed by the compiler) unless kAhead
        if (kAhead) {
            if (t + 1 < nstages) load_frags(an, t + 1);
        } else {
            load_frags(a, t);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < nstages) load_stage(t + 1);
        __builtin_amdgcn_sched_barrier(0);
        lds_barrier();
#pragma unroll
        for (int ks = 0; ks < KSW; ++ks) {
            const int s = wk * KSW + ks;
            uint4 b[RBW][NS];
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                for (int h = 0; h < NS; ++h) {
                    const int row = (wr * RBW + rb) * 32 + (lane & 31);
                    b[rb][h] = *reinterpret_cast<const uint4 *>(
                        buf + (h * kRows + row) * kPPitch + s * 32 + (lane >> 5) * 16);
                }
#pragma unroll
            for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb) mfma_split<NS>(a[ks][cb], b[rb], acc[cb][rb]);
        }
        if (kAhead && t + 1 < nstages) {
#pragma unroll
            for (int ks = 0; ks < KSW; ++ks)
#pragma unroll
                for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
                    for (int h = 0; h < NS; ++h) a[ks][cb][h] = an[ks][cb][h];
        }
    }
    if (WK == 2) {  // add the two halves of the reduction: wk = 1 hands over through LDS
        __syncthreads();
        float *red = reinterpret_cast<float *>(lds);
        const int slot = wr * WC + wc;  // WK == 2 => WC * WR == 2
        if (wk == 1) {
#pragma unroll
            for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        red[((slot * CBW * RBW + cb * RBW + rb) * 16 + v) * 64 + lane] = acc[cb][rb][v];
        }
        __syncthreads();
        if (wk == 1) return;
#pragma unroll
        for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    acc[cb][rb][v] += red[((slot * CBW * RBW + cb * RBW + rb) * 16 + v) * 64 + lane];
    }
#pragma unroll
    for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
            const int64_t i = i0 + (wr * RBW + rb) * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int c = (wc * CBW + cb) * 32 + d_row(v, lane);
                if (c < r && i < m) out[(int64_t)c * m + i] = acc[cb][rb][v];
            }
        }
}

// ---------------------------------------------------------------------------------------------
// P phase at 8 basis blocks (128 < r <= 256), where a stage of matrix-core work is about as long
// as a round trip to HBM and a single wavefront per SIMD cannot hide one behind the other.  The
// workgroup has 8 wavefronts with two roles.  Wavefronts 4..7 (producers) stream delta: stage s
// lives in register set s & 1, is split into bf16 pieces and laid down in LDS buffer s & 1 one
// stage before it is used, and its set is refilled at once with stage s + 2, so that every
// request has two stages of time to come back.  Wavefronts 0..3 (consumers) own WC x WR blocks of
// the output, fetch their basis fragments through L2 two or four k-steps ahead (their load
// counter never waits for HBM) and keep the matrix cores busy on the buffer the producers filled
// last.  One
// LDS-only barrier per stage for all eight.  Loads past the matrix or past the last stage are
// clamped to a valid address and zeroed / never read, which keeps both loops free of branches.
// ---------------------------------------------------------------------------------------------
constexpr int kWs = 512;  // threads of the two-role workgroup

// NS == 1 is the fp16 form (one product per block instead of three): the producers multiply
// delta by 2^kF16DeltaShift and record its largest magnitude in *amax_record, the consumers undo
// the scales through out_scale.  `guard` (NS >= 2) makes the launch a stand-by: it returns at
// once if the fp16 launch before it saw its operands in range.
template <int NS, int CBW, int WC, int WR, int RB>
__global__ __launch_bounds__(kWs) void project_p_ws_kernel(PtrPack<const float *> deltas,
                                                           const uint4 *__restrict__ afrags,
                                                           PtrPack<float *> outs, int64_t m,
                                                           int64_t n, int r,
                                                           uint32_t *__restrict__ amax_record,
                                                           const float *__restrict__ out_scale,
                                                           const uint32_t *__restrict__ guard) {
    constexpr int CB = CBW * WC;
    constexpr int RBW = RB / WR;
    constexpr int kRows = 32 * RB;
    constexpr int kVec = kRows * 16 / kW;  // float4 per producer thread and stage
    static_assert(WC * WR == 4, "four consumer wavefronts");
    constexpr int kBuf = NS * kRows * kPPitch;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    if (guard != nullptr && f16_range_ok(*guard)) return;  // uniform over the launch
    const float *__restrict__ delta = deltas.p[blockIdx.y];
    float *__restrict__ out = outs.p[blockIdx.y];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t i0 = (int64_t)blockIdx.x * kRows;
    const int64_t nstages = (n + 63) / 64;

    if (wave >= 4) {  // ---------------------------------------------------------- producers
        const int tid = threadIdx.x - kW;
        float amax = 0.f;  // NS == 1: largest |delta| this thread has laid down
        auto load_stage = [&](float4 (&set)[kVec], int64_t t) {
            const int64_t tc = t < nstages ? t : nstages - 1;
#pragma unroll
            for (int u = 0; u < kVec; ++u) {
                const int idx = tid + kW * u;
                const int row = idx >> 4, c4 = idx & 15;
                const int64_t j = tc * 64 + c4 * 4;
                const bool ok = i0 + row < m && j < n;
                // the value of a clamped load is discarded when the stage is laid down, not
                // here: touching it now would wait for the request just made
                set[u] = stream_load4(ok ? delta + (i0 + row) * n + j : delta);
            }
        };
        auto store_stage = [&](const float4 (&set)[kVec], unsigned char *buf, int64_t t) {
#pragma unroll
            for (int u = 0; u < kVec; ++u) {
                const int idx = tid + kW * u;
                const int row = idx >> 4, c4 = idx & 15;
                const bool ok = i0 + row < m && t * 64 + c4 * 4 < n;
                float4 x = make_float4(ok ? set[u].x : 0.f, ok ? set[u].y : 0.f,
                                       ok ? set[u].z : 0.f, ok ? set[u].w : 0.f);
                if constexpr (NS == 1) {
                    amax = fmaxf(fmaxf(amax, fmaxf(fabsf(x.x), fabsf(x.y))),
                                 fmaxf(fabsf(x.z), fabsf(x.w)));
                    constexpr float kUp = (float)(1 << kF16DeltaShift);
                    x = make_float4(x.x * kUp, x.y * kUp, x.z * kUp, x.w * kUp);
                }
                uint32_t lo[NS], hi[NS];
                split2<NS>(x.x, x.y, lo);
                split2<NS>(x.z, x.w, hi);
#pragma unroll
                for (int h = 0; h < NS; ++h)
                    *reinterpret_cast<uint2 *>(buf + (h * kRows + row) * kPPitch + c4 * 8) =
                        make_uint2(lo[h], hi[h]);
            }
        };
        // one step: lay down stage `stage` (held in `set`) for the consumers' next iteration
        // while they work on the stage before it, then refill the set two stages further on
        auto step = [&](float4 (&set)[kVec], int64_t stage, bool refill) {
            store_stage(set, lds + (stage & 1) * kBuf, stage);
            if (refill) load_stage(set, stage + 2);
            lds_barrier();
            // nothing of the next step moves above the barrier: splitting its set earlier would
            // wait for requests that are younger than they should be
            __builtin_amdgcn_sched_barrier(0);
        };
        float4 set0[kVec], set1[kVec];
        load_stage(set0, 0);
        load_stage(set1, 1);
        step(set0, 0, true);
        // two stages per trip, no way round the second inside the loop: the compiler's wait
        // counts at the loop head then see one order of outstanding requests only.  (Four sets
        // and four stages of distance measured no faster.)
        int64_t t = 0;
        for (; t + 1 < nstages; t += 2) {
            step(set1, t + 1, true);
            step(set0, t + 2, true);
        }
        // an odd number of stages: the consumers' last iteration needs its barrier
        if (t < nstages) step(set1, t + 1, false);
        if constexpr (NS == 1) record_amax(amax, amax_record);
        return;
    }
    // -------------------------------------------------------------------------------- consumers
    const int wc = wave % WC, wr = wave / WC;
    f32x16_t acc[CBW][RBW];
#pragma unroll
    for (int a = 0; a < CBW; ++a)
#pragma unroll
        for (int b = 0; b < RBW; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    // fragments of global k-step g (4 per stage) in ring position g % AD: requested two k-steps
    // ahead, or a whole stage ahead where that is at most 8 registers per position (one fp16
    // piece, or one basis block per wavefront).  There the matrix-core work of two k-steps is
    // shorter than a trip to L2 and the consumers, hence the stage barrier, waited for fragments:
    // 4 - 10 % on the kernel at rank 64, 4 - 7 % in the fp16 form at ranks 192 and 256.  With two
    // blocks of two bf16 pieces the matrix cores set the pace and the deeper ring gains nothing.
    constexpr int AD = CBW * NS <= 2 ? 4 : 2;
    uint4 a[AD][CBW][NS];
    const int64_t gmax = nstages * 4 - 1;
    auto load_frags = [&](int64_t g, int pos) {
        const int64_t gc = g < gmax ? g : gmax;
#pragma unroll
        for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
            for (int h = 0; h < NS; ++h)
                a[pos][cb][h] = afrags[((gc * CB + wc * CBW + cb) * NS + h) * 64 + lane];
    };
#pragma unroll
    for (int g = 0; g < AD; ++g) load_frags(g, g);
    lds_barrier();
    for (int64_t t = 0; t < nstages; ++t) {
        const unsigned char *buf = lds + (t & 1) * kBuf;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint4 b[RBW][NS];
#pragma unroll
            for (int rb = 0; rb < RBW; ++rb)
#pragma unroll
                for (int h = 0; h < NS; ++h) {
                    const int row = (wr * RBW + rb) * 32 + (lane & 31);
                    b[rb][h] = *reinterpret_cast<const uint4 *>(
                        buf + (h * kRows + row) * kPPitch + ks * 32 + (lane >> 5) * 16);
                }
#pragma unroll
            for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
                for (int rb = 0; rb < RBW; ++rb)
                    mfma_split<NS>(a[ks % AD][cb], b[rb], acc[cb][rb]);
            // requested here and nowhere later: AD k-steps of matrix-core work to come back
            load_frags(t * 4 + ks + AD, ks % AD);
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();
    }
#pragma unroll
    for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
        for (int rb = 0; rb < RBW; ++rb) {
            const int64_t i = i0 + (wr * RBW + rb) * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int c = (wc * CBW + cb) * 32 + d_row(v, lane);
                if (c < r && i < m)
                    out[(int64_t)c * m + i] = NS == 1 ? acc[cb][rb][v] * out_scale[c] : acc[cb][rb][v];
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Q phase:  Q_k[j][c] = sum_i delta_k[i][j] P_hat[c][i].
// Wavefront: 32 JB columns x all CB basis blocks over its own range of rows.  The B operand
// (N = column, reduction down the column) is loaded straight from HBM into the operand layout:
// lane (x, half) reads the JB consecutive columns j0 + JB x .. of the rows i0 + 8 half + e,
// e = 0..7, and column JB x + q feeds MFMA block q (the column blocks are interleaved, which an
// MFMA does not care about), so one load instruction covers 2 rows x 128 JB contiguous bytes.
// The 4 wavefronts of a workgroup take consecutive quarters of the workgroup's rows and are added
// in wavefront order at the end; blockIdx.z splits the rows further into slabs.
// ---------------------------------------------------------------------------------------------
template <int JB> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef float2 type; };
template <> struct VecOf<4> { typedef float4 type; };

template <int JB>
__device__ __forceinline__ void vec_to_array(const typename VecOf<JB>::type &v, float (&out)[JB]);
template <>
__device__ __forceinline__ void vec_to_array<1>(const float &v, float (&out)[1]) { out[0] = v; }
template <>
__device__ __forceinline__ void vec_to_array<2>(const float2 &v, float (&out)[2]) {
    out[0] = v.x; out[1] = v.y;
}
template <>
__device__ __forceinline__ void vec_to_array<4>(const float4 &v, float (&out)[4]) {
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}

// Used for one basis block (r <= 32); from two blocks on project_q_ws_kernel below (at two
// blocks this kernel needs 326 registers, one wavefront per SIMD: 4.8 - 5.5 TB/s on the large
// shapes against 4.9 - 6.0).
template <int JB>
__device__ __forceinline__ typename VecOf<JB>::type stream_load_vec(const float *p);
template <>
__device__ __forceinline__ float stream_load_vec<1>(const float *p) {
    return __builtin_nontemporal_load(p);
}
template <>
__device__ __forceinline__ float2 stream_load_vec<2>(const float *p) {
    typedef float nt_f32x2 __attribute__((ext_vector_type(2)));
    const nt_f32x2 v = __builtin_nontemporal_load(reinterpret_cast<const nt_f32x2 *>(p));
    return make_float2(v.x, v.y);
}
template <>
__device__ __forceinline__ float4 stream_load_vec<4>(const float *p) {
    return stream_load4(p);
}

template <int NS, int CB, int JB, int DEPTH>
__global__ __launch_bounds__(kW) void project_q_mfma_kernel(PtrPack<const float *> deltas,
                                                            const uint4 *__restrict__ afrags,
                                                            PtrPack<float *> outs, int64_t m,
                                                            int64_t n, int r,
                                                            int64_t ksteps_per_wave,
                                                            int64_t slab_stride) {
    __shared__ float red[CB * JB * 16 * 64];
    const float *__restrict__ delta = deltas.p[blockIdx.y];
    float *__restrict__ out = outs.p[blockIdx.y] + (int64_t)blockIdx.z * slab_stride;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t jcol = (int64_t)blockIdx.x * (32 * JB) + JB * (lane & 31);
    const bool col_ok = jcol < n;  // n is a multiple of 16: the JB columns are in or out together
    const int64_t s_begin = ((int64_t)blockIdx.z * 4 + wave) * ksteps_per_wave;
    const int64_t s_end = s_begin + ksteps_per_wave;  // a multiple of DEPTH k-steps

    f32x16_t acc[CB][JB];
#pragma unroll
    for (int a = 0; a < CB; ++a)
#pragma unroll
        for (int b = 0; b < JB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    float breg[DEPTH][8][JB];
    auto load_kstep = [&](int d, int64_t s) {
        const int64_t ibase = s * 16 + (lane >> 5) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
#pragma unroll
            for (int q = 0; q < JB; ++q) breg[d][e][q] = 0.f;
            if (ibase + e < m && col_ok)
                vec_to_array<JB>(stream_load_vec<JB>(delta + (ibase + e) * n + jcol), breg[d][e]);
        }
    };
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) load_kstep(d, s_begin + d);
    for (int64_t s = s_begin; s < s_end; s += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            uint4 a[CB][NS];
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int h = 0; h < NS; ++h)
                    a[cb][h] = afrags[(((s + d) * CB + cb) * NS + h) * 64 + lane];
            uint4 b[JB][NS];
#pragma unroll
            for (int q = 0; q < JB; ++q) {
                float x[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = breg[d][e][q];
                split8<NS>(x, b[q]);
            }
            if (s + d + DEPTH < s_end) load_kstep(d, s + d + DEPTH);
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int q = 0; q < JB; ++q) mfma_split<NS>(a[cb], b[q], acc[cb][q]);
        }
    }
    // wavefronts 3, 2, 1 hand their sums to wavefront 0, in that order
    for (int w = 3; w >= 1; --w) {
        if (wave == w) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int q = 0; q < JB; ++q)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        red[((cb * JB + q) * 16 + v) * 64 + lane] = acc[cb][q][v];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int q = 0; q < JB; ++q)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[cb][q][v] += red[((cb * JB + q) * 16 + v) * 64 + lane];
        }
        __syncthreads();
    }
    if (wave != 0 || !col_ok) return;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int c = cb * 32 + d_row(v, lane);
            if (c < r) {
#pragma unroll
                for (int q = 0; q < JB; ++q) out[(int64_t)c * n + jcol + q] = acc[cb][q][v];
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Reconstruction  delta_hat[i][j] = sum_c P_hat[c][i] Q_bar[c][j]  with fused consumers.
// Workgroup: 32 rows x 256 columns per iteration, swept along j; wavefront w owns the 64 columns
// 64 w .. 64 w + 63 (two 32 x 32 MFMA blocks; A = P_hat fragments with M = i, B = Q_bar fragments
// with N = j).  The accumulators (lane = column, register = row) go through a wavefront-private
// LDS tile so that every access to a matrix element is a 16-byte vector and a wavefront
// instruction covers 4 rows x 256 contiguous bytes, the same shape as a plain streaming kernel:
//   out            : delta_hat is written
//   K > 0          : e_k <- e_k - delta_hat                      (error buffers of Alg. 2)
//   tl_on          : e_k <- (theta - theta_l,k) + e_k            (next pseudo-gradient)
//   apply          : v <- mu v + delta_hat; theta <- theta - lr (delta_hat + mu v)   (OuterOpt)
// ---------------------------------------------------------------------------------------------
constexpr int kRPitch = 64 + 4;  // floats per LDS tile row

template <int NS>
__global__ __launch_bounds__(kW) void reconstruct_mfma_kernel(
    const uint4 *__restrict__ pfrags, const uint4 *__restrict__ qfrags, ReconEpilogue ep,
    int64_t m, int64_t n, int64_t cols_per_wg, int KS) {
    __shared__ __attribute__((aligned(16))) float tile[4][32][kRPitch];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t ib = blockIdx.y;
    const int64_t jbegin = (int64_t)blockIdx.x * cols_per_wg;
    int64_t jend = jbegin + cols_per_wg;
    if (jend > n) jend = n;
    const int64_t nblk = (n + 31) >> 5;
    const int prow = lane >> 4, pc4 = lane & 15;  // epilogue: 4 rows x 16 float4 per instruction

    for (int64_t jt0 = jbegin; jt0 < jend; jt0 += 256) {  // uniform over the workgroup
        const int64_t jt = jt0 + wave * 64;
        f32x16_t d[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) d[nb][v] = 0.f;
        if (jt < jend) {
            const int64_t jb0 = jt >> 5;
            const bool two = jb0 + 1 < nblk;
            for (int s = 0; s < KS; ++s) {
                uint4 a[NS], b0[NS], b1[NS];
#pragma unroll
                for (int h = 0; h < NS; ++h) {
                    a[h] = pfrags[((ib * KS + s) * NS + h) * 64 + lane];
                    b0[h] = qfrags[((jb0 * KS + s) * NS + h) * 64 + lane];
                    b1[h] = two ? qfrags[(((jb0 + 1) * KS + s) * NS + h) * 64 + lane]
                                : make_uint4(0u, 0u, 0u, 0u);
                }
                mfma_split<NS>(a, b0, d[0]);
                mfma_split<NS>(a, b1, d[1]);
            }
        }
        __syncthreads();  // the previous iteration's readers are done with the tile
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                tile[wave][d_row(v, lane)][nb * 32 + (lane & 31)] = d[nb][v];
        __syncthreads();
        const int64_t j = jt + pc4 * 4;
        const bool col_ok = jt < jend && j < n;
        for (int pass = 0; pass < 8; ++pass) {
            const int row = pass * 4 + prow;
            const int64_t i = ib * 32 + row;
            // outside the matrix a lane reads element 0 (dropped) instead of skipping its loads
            // behind a per-lane condition, and stores nothing
            const bool ok = col_ok && i < m;
            const int64_t off = ok ? i * n + j : 0;
            const float4 dv = *reinterpret_cast<const float4 *>(&tile[wave][row][pc4 * 4]);
            if (ep.out) {
                if (ok) stream_store4(ep.out + off, dv);
            }
            float4 tv = make_float4(0.f, 0.f, 0.f, 0.f), vv = tv;
            if (ep.tl_on || ep.apply) tv = stream_load4(ep.theta + off);
            if (ep.apply) vv = stream_load4(ep.vel + off);
            for (int k0 = 0; k0 < ep.K; k0 += 4) {
                float4 x[4], l[4];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    if (k0 + kk < ep.K) {
                        x[kk] = stream_load4(ep.ef.p[k0 + kk] + off);
                        if (ep.tl_on) {
                            if (ep.tl_bf16) {
                                const uint2 bits = stream_load2(
                                    reinterpret_cast<const uint16_t *>(ep.tl.p[k0 + kk]) + off);
                                l[kk] = make_float4(__uint_as_float(bits.x << 16),
                                                    __uint_as_float(bits.x & 0xFFFF0000u),
                                                    __uint_as_float(bits.y << 16),
                                                    __uint_as_float(bits.y & 0xFFFF0000u));
                            } else {
                                l[kk] = stream_load4(
                                    reinterpret_cast<const float *>(ep.tl.p[k0 + kk]) + off);
                            }
                        }
                    }
                }
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    if (k0 + kk < ep.K) {
                        float4 e;
                        e.x = x[kk].x - dv.x; e.y = x[kk].y - dv.y;
                        e.z = x[kk].z - dv.z; e.w = x[kk].w - dv.w;
                        if (ep.tl_on) {
                            e.x = (tv.x - l[kk].x) + e.x; e.y = (tv.y - l[kk].y) + e.y;
                            e.z = (tv.z - l[kk].z) + e.z; e.w = (tv.w - l[kk].w) + e.w;
                        }
                        if (ok) stream_store4(ep.ef.p[k0 + kk] + off, e);
                    }
                }
            }
            if (ep.apply && ok) {
                float4 vn, tn;
                vn.x = fmaf(ep.mu, vv.x, dv.x); vn.y = fmaf(ep.mu, vv.y, dv.y);
                vn.z = fmaf(ep.mu, vv.z, dv.z); vn.w = fmaf(ep.mu, vv.w, dv.w);
                tn.x = fmaf(-ep.lr, fmaf(ep.mu, vn.x, dv.x), tv.x);
                tn.y = fmaf(-ep.lr, fmaf(ep.mu, vn.y, dv.y), tv.y);
                tn.z = fmaf(-ep.lr, fmaf(ep.mu, vn.z, dv.z), tv.z);
                tn.w = fmaf(-ep.lr, fmaf(ep.mu, vn.w, dv.w), tv.w);
                stream_store4(ep.vel + off, vn);
                stream_store4(ep.theta + off, tn);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The whole pass between two compressions, fused with the P phase of the next one (outer step
// t >= 2), for up to KC workers:
//   d        = P_hat_prev Q_bar_prev^T             (tile by tile, never written)
//   e_k      = delta_k - d ;  delta_k = (theta - theta_l,k) + e_k     -> stored over delta_k
//   P_k     += delta_k Q_in                        (accumulated while the tile is on chip)
//   apply    : v <- mu v + d ; theta <- theta - lr (d + mu v)
// Same tiling as the reconstruction kernel (32 rows x 256 columns per iteration, wavefront w owns
// 64 columns).  After the elementwise step the new delta_k tile is written to LDS as bf16 pieces
// in the layout of the P-phase kernel (row-major, reduction index contiguous) and multiplied with
// the basis fragments of its 64 columns: delta is read from HBM once for all of this.  A
// workgroup leaves the partial P_k of its rows and column range in slab blockIdx.x; the slabs of
// a row block are added afterwards in slab order.
// ---------------------------------------------------------------------------------------------
// LDS written by some lanes of a wavefront and read by others: the data share unit executes one
// wavefront's instructions in order, so only the compiler has to be kept from reordering.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int NS, int CB, int KC, bool TLBF16>
__global__ __launch_bounds__(kW) void round_mfma_kernel(
    const uint4 *__restrict__ pfrags, const uint4 *__restrict__ qfrags, int KS,
    const uint4 *__restrict__ bfrags, ReconEpilogue ep, PtrPack<float *> pslab, int64_t m,
    int64_t n, int r, int64_t cols_per_wg, int64_t slab_stride) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int kTileBytes = 32 * kRPitch * 4;      // fp32 staging tile of one wavefront
    constexpr int kBBytes = NS * 32 * kPPitch;        // bf16 pieces of one wavefront's delta tile
    constexpr bool kBasisInLds = NS == 2 && CB <= 2;  // basis fragments of the 64 columns staged
    constexpr int kBasisBytes = kBasisInLds ? 4 * CB * NS * 1024 : 0;
    float *tile = reinterpret_cast<float *>(smem) + (threadIdx.x >> 6) * (32 * kRPitch);
    unsigned char *btile = smem + 4 * kTileBytes + (threadIdx.x >> 6) * kBBytes;
    uint4 *basis_lds = reinterpret_cast<uint4 *>(smem + 4 * kTileBytes + 4 * kBBytes +
                                                 (threadIdx.x >> 6) * kBasisBytes);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t ib = blockIdx.y;
    const int64_t jbegin = (int64_t)blockIdx.x * cols_per_wg;
    int64_t jend = jbegin + cols_per_wg;
    if (jend > n) jend = n;
    const int64_t nblk = (n + 31) >> 5;
    const int prow = lane >> 4, pc4 = lane & 15;
    const int64_t row0 = ib * 32 + prow;  // pass p covers row row0 + 4 p
    typedef typename std::conditional<TLBF16, uint2, float4>::type traw_t;

    f32x16_t acc[KC][CB];
#pragma unroll
    for (int k = 0; k < KC; ++k)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[k][cb][v] = 0.f;

    // operands of the item (column tile, worker) in flight
    float4 x[8], tv[8], vv[8];
    traw_t lraw[8];
    auto issue = [&](int64_t jt, int k, bool with_theta, bool with_vel) {
        const int64_t j = jt + pc4 * 4;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            // outside the matrix: element 0 instead (what comes back is never used: the new
            // delta is forced to zero there and nothing is stored), so that no lane branches
            const bool okp = j < n && row0 + 4 * p < m;
            const int64_t off = okp ? (row0 + 4 * p) * n + j : 0;
            x[p] = stream_load4(ep.ef.p[k] + off);
            if constexpr (TLBF16)
                lraw[p] = stream_load2(reinterpret_cast<const uint16_t *>(ep.tl.p[k]) + off);
            else
                lraw[p] = stream_load4(reinterpret_cast<const float *>(ep.tl.p[k]) + off);
            if (with_theta) tv[p] = stream_load4(ep.theta + off);
            if (with_vel) vv[p] = stream_load4(ep.vel + off);
        }
    };
    const int Kw = ep.K;
    // This wavefront's tiles are the columns jw + 256 t, t = 0 .. nw - 1.  They are visited in
    // rotated order: the workgroups of a launch start together, and without the rotation all
    // of them would sweep the same columns of different rows at the same time, rows whose
    // distance in memory is the same multiple of a power of two for the common matrix widths.
    const int64_t jw = jbegin + wave * 64;
    const int64_t nw = jw < jend ? (jend - jw + 255) >> 8 : 0;
    // Starting tile: groups of 8 consecutive row blocks start a quarter of the range apart
    // (4 starting points).  Measured against a start of ib mod nw (every row block its own):
    // 5 - 6 % faster on the 8192-column shapes, no difference at 28672 columns; with 8 or 16
    // starting points, or groups of 1 or 2 row blocks, the gain is smaller or gone.
    const int64_t pp = nw < 4 ? nw : 4;
    const int64_t shift = nw > 0 ? ((ib >> 3) % pp) * nw / pp : 0;
    auto tile_at = [&](int64_t i) {
        const int64_t t = i + shift;
        return jw + ((t >= nw ? t - nw : t) << 8);
    };
    if (nw > 0) issue(tile_at(0), 0, true, ep.apply && Kw == 1);
    for (int64_t it = 0; it < nw; ++it) {
        const int64_t jt = tile_at(it);
        // ---- d = P_hat_prev Q_bar_prev^T for this wavefront's 32 x 64 tile
        f32x16_t d[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) d[nb][v] = 0.f;
        {
            const int64_t jb0 = jt >> 5;
            const bool two = jb0 + 1 < nblk;
            for (int s = 0; s < KS; ++s) {
                uint4 a[NS], b0[NS], b1[NS];
#pragma unroll
                for (int h = 0; h < NS; ++h) {
                    a[h] = pfrags[((ib * KS + s) * NS + h) * 64 + lane];
                    b0[h] = qfrags[((jb0 * KS + s) * NS + h) * 64 + lane];
                    b1[h] = two ? qfrags[(((jb0 + 1) * KS + s) * NS + h) * 64 + lane]
                                : make_uint4(0u, 0u, 0u, 0u);
                }
                mfma_split<NS>(a, b0, d[0]);
                mfma_split<NS>(a, b1, d[1]);
            }
        }
        wave_lds_sync();  // earlier readers of the staging tile and of the basis are done
        if (kBasisInLds) {  // this tile's basis fragments: 4 k-steps x CB blocks x NS pieces
#pragma unroll
            for (int f = 0; f < 4 * CB * NS; ++f)
                basis_lds[f * 64 + lane] = bfrags[((jt >> 4) * CB * NS + f) * 64 + lane];
        }
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                tile[d_row(v, lane) * kRPitch + nb * 32 + (lane & 31)] = d[nb][v];
        wave_lds_sync();
        float4 dv[8];
#pragma unroll
        for (int p = 0; p < 8; ++p)
            dv[p] = *reinterpret_cast<const float4 *>(&tile[(p * 4 + prow) * kRPitch + pc4 * 4]);
        const int64_t j = jt + pc4 * 4;
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            if (k < Kw) {
                const bool last = k == Kw - 1;
                float *__restrict__ e = ep.ef.p[k];
                wave_lds_sync();  // the previous item's fragments have been read
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const bool okp = j < n && row0 + 4 * p < m;
                    const int64_t off = (row0 + 4 * p) * n + j;
                    float4 l;
                    if (TLBF16) {
                        const uint2 bits = *reinterpret_cast<const uint2 *>(&lraw[p]);
                        l = make_float4(__uint_as_float(bits.x << 16),
                                        __uint_as_float(bits.x & 0xFFFF0000u),
                                        __uint_as_float(bits.y << 16),
                                        __uint_as_float(bits.y & 0xFFFF0000u));
                    } else {
                        l = *reinterpret_cast<const float4 *>(&lraw[p]);
                    }
                    float4 g;
                    g.x = (tv[p].x - l.x) + (x[p].x - dv[p].x);
                    g.y = (tv[p].y - l.y) + (x[p].y - dv[p].y);
                    g.z = (tv[p].z - l.z) + (x[p].z - dv[p].z);
                    g.w = (tv[p].w - l.w) + (x[p].w - dv[p].w);
                    if (okp) {
                        stream_store4(e + off, g);
                    } else {
                        g = make_float4(0.f, 0.f, 0.f, 0.f);
                    }
                    uint32_t lo[NS], hi[NS];
                    split2<NS>(g.x, g.y, lo);
                    split2<NS>(g.z, g.w, hi);
#pragma unroll
                    for (int h = 0; h < NS; ++h)
                        *reinterpret_cast<uint2 *>(btile + (h * 32 + p * 4 + prow) * kPPitch +
                                                   pc4 * 8) = make_uint2(lo[h], hi[h]);
                    if (last && ep.apply && okp) {
                        float4 vn, tn;
                        vn.x = fmaf(ep.mu, vv[p].x, dv[p].x); vn.y = fmaf(ep.mu, vv[p].y, dv[p].y);
                        vn.z = fmaf(ep.mu, vv[p].z, dv[p].z); vn.w = fmaf(ep.mu, vv[p].w, dv[p].w);
                        tn.x = fmaf(-ep.lr, fmaf(ep.mu, vn.x, dv[p].x), tv[p].x);
                        tn.y = fmaf(-ep.lr, fmaf(ep.mu, vn.y, dv[p].y), tv[p].y);
                        tn.z = fmaf(-ep.lr, fmaf(ep.mu, vn.z, dv[p].z), tv[p].z);
                        tn.w = fmaf(-ep.lr, fmaf(ep.mu, vn.w, dv[p].w), tv[p].w);
                        stream_store4(ep.vel + off, vn);
                        stream_store4(ep.theta + off, tn);
                    }
                }
                // operands of the next item, in flight while this one is multiplied
                if (!last) {
                    issue(jt, k + 1, false, ep.apply && k + 1 == Kw - 1);
                } else if (it + 1 < nw) {
                    issue(tile_at(it + 1), 0, true, ep.apply && Kw == 1);
                }
                wave_lds_sync();
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    uint4 b[NS];
#pragma unroll
                    for (int h = 0; h < NS; ++h)
                        b[h] = *reinterpret_cast<const uint4 *>(
                            btile + (h * 32 + (lane & 31)) * kPPitch + s * 32 + (lane >> 5) * 16);
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        uint4 a[NS];
#pragma unroll
                        for (int h = 0; h < NS; ++h) {
                            if (kBasisInLds)
                                a[h] = basis_lds[((s * CB + cb) * NS + h) * 64 + lane];
                            else
                                a[h] = bfrags[((((jt >> 4) + s) * CB + cb) * NS + h) * 64 + lane];
                        }
                        mfma_split<NS>(a, b, acc[k][cb]);
                    }
                }
            }
        }
    }
    // add the four wavefronts' partial P_k (wavefronts 3, 2, 1 hand over to 0, in that order)
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);
    for (int w = 3; w >= 1; --w) {
        if (wave == w) {
#pragma unroll
            for (int k = 0; k < KC; ++k)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        red[((k * CB + cb) * 16 + v) * 64 + lane] = acc[k][cb][v];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int k = 0; k < KC; ++k)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[k][cb][v] += red[((k * CB + cb) * 16 + v) * 64 + lane];
        }
        __syncthreads();
    }
    if (wave != 0) return;
    const int64_t i = ib * 32 + (lane & 31);
    if (i >= m) return;
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        if (k < Kw) {
            float *__restrict__ out = pslab.p[k] + (int64_t)blockIdx.x * slab_stride;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int c = cb * 32 + d_row(v, lane);
                    if (c < r) out[(int64_t)c * m + i] = acc[k][cb][v];
                }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Q phase for 4 or 8 basis blocks in the two-role form of project_p_ws_kernel.  A workgroup owns
// 128 columns and a range of rows, swept in stages of 64 rows (4 k-steps).  Producer thread
// (column quad c4, row group rg) requests 8 rows x 4 columns per stage -- one instruction of a
// wavefront covers 2 rows x 512 bytes -- and holds, for each of its 4 columns, exactly the 8
// reduction-consecutive values one lane feeds to the matrix cores: it splits them into bf16
// pieces and writes them to LDS in operand order, so that a consumer fetches one 16 x 32 operand
// block of one piece as 1 KB of consecutive LDS.  The consumers form a WCB x (4 / WCB) grid:
// wavefront w owns the CBW basis blocks of group w % WCB and WCB of the four 32-column blocks.
// Register sets, buffers, barriers and clamping as in the P kernel.
// ---------------------------------------------------------------------------------------------
template <int NS, int CBW, int WCB>
__global__ __launch_bounds__(kWs) void project_q_ws_kernel(PtrPack<const float *> deltas,
                                                           const uint4 *__restrict__ afrags,
                                                           PtrPack<float *> outs, int64_t m,
                                                           int64_t n, int r, int64_t ksteps_per_wg,
                                                           int64_t slab_stride,
                                                           uint32_t *__restrict__ amax_record,
                                                           const float *__restrict__ out_scale,
                                                           const uint32_t *__restrict__ guard) {
    constexpr int CB = WCB * CBW;
    constexpr int QW = WCB;               // column blocks per consumer: 4 / (4 / WCB)
    constexpr int kBuf = 16 * NS * 1024;  // 4 k-steps x 4 column blocks x NS pieces x 1 KB
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    if (guard != nullptr && f16_range_ok(*guard)) return;  // uniform over the launch
    const float *__restrict__ delta = deltas.p[blockIdx.y];
    float *__restrict__ out = outs.p[blockIdx.y] + (int64_t)blockIdx.z * slab_stride;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t j0 = (int64_t)blockIdx.x * 128;
    const int64_t s_begin = (int64_t)blockIdx.z * ksteps_per_wg;  // a multiple of 4
    const int64_t nstages = ksteps_per_wg >> 2;

    if (wave >= 4) {  // ---------------------------------------------------------- producers
        const int tid = threadIdx.x - kW;
        const int c4 = tid & 31, rg = tid >> 5;
        const bool col_ok = j0 + c4 * 4 < n;
        float amax = 0.f;  // NS == 1: largest |delta| this thread has laid down
        auto load_stage = [&](float4 (&set)[8], int64_t t) {
            const int64_t tc = t < nstages ? t : nstages - 1;
            const int64_t i0 = (s_begin + 4 * tc) * 16 + rg * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool ok = col_ok && i0 + e < m;
                set[e] = stream_load4(ok ? delta + (i0 + e) * n + j0 + c4 * 4 : delta);
            }
        };
        auto store_stage = [&](const float4 (&set)[8], unsigned char *buf, int64_t t) {
            const int64_t i0 = (s_begin + 4 * t) * 16 + rg * 8;
            float v[4][8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool ok = col_ok && i0 + e < m;
                v[0][e] = ok ? set[e].x : 0.f;
                v[1][e] = ok ? set[e].y : 0.f;
                v[2][e] = ok ? set[e].z : 0.f;
                v[3][e] = ok ? set[e].w : 0.f;
            }
            if constexpr (NS == 1) {
                constexpr float kUp = (float)(1 << kF16DeltaShift);
#pragma unroll
                for (int x = 0; x < 4; ++x)
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        amax = fmaxf(amax, fabsf(v[x][e]));
                        v[x][e] *= kUp;
                    }
            }
            // operand block (k-step rg / 2, column block c4 / 8), lane (rg % 2) 32 + column
            // (the two low bits of the lane slot are swizzled so that the 16 lanes of one LDS
            // pass, which differ in c4, fall on 16 different bank groups; a consumer reads the
            // 64 slots of a block in the same permutation)
            unsigned char *blk = buf + ((rg >> 1) * 4 + (c4 >> 3)) * NS * 1024 +
                                 ((rg & 1) * 32 + (c4 & 7) * 4) * 16;
            const int sw = (((c4 >> 2) & 1) << 1) | ((c4 >> 3) & 1);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                uint4 pieces[NS];
                split8<NS>(v[x], pieces);
#pragma unroll
                for (int h = 0; h < NS; ++h)
                    *reinterpret_cast<uint4 *>(blk + h * 1024 + (x ^ sw) * 16) = pieces[h];
            }
        };
        auto step = [&](float4 (&set)[8], int64_t stage, bool refill) {
            store_stage(set, lds + (stage & 1) * kBuf, stage);
            if (refill) load_stage(set, stage + 2);
            lds_barrier();
            __builtin_amdgcn_sched_barrier(0);
        };
        float4 set0[8], set1[8];
        load_stage(set0, 0);
        load_stage(set1, 1);
        step(set0, 0, true);
        int64_t t = 0;
        for (; t + 1 < nstages; t += 2) {
            step(set1, t + 1, true);
            step(set0, t + 2, true);
        }
        if (t < nstages) step(set1, t + 1, false);
        if constexpr (NS == 1) record_amax(amax, amax_record);
        return;
    }
    // -------------------------------------------------------------------------------- consumers
    const int wcb = wave % WCB, wq = wave / WCB;
    f32x16_t acc[CBW][QW];
#pragma unroll
    for (int a = 0; a < CBW; ++a)
#pragma unroll
        for (int b = 0; b < QW; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    constexpr int AD = CBW * NS <= 2 ? 4 : 2;  // as in project_p_ws_kernel
    uint4 a[AD][CBW][NS];                      // fragments of k-step g in ring position g % AD
    const int64_t gmax = s_begin + ksteps_per_wg - 1;
    auto load_frags = [&](int64_t g, int pos) {
        const int64_t gc = g < gmax ? g : gmax;
#pragma unroll
        for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
            for (int h = 0; h < NS; ++h)
                a[pos][cb][h] = afrags[((gc * CB + wcb * CBW + cb) * NS + h) * 64 + lane];
    };
#pragma unroll
    for (int g = 0; g < AD; ++g) load_frags(s_begin + g, g);
    lds_barrier();
    for (int64_t t = 0; t < nstages; ++t) {
        const unsigned char *buf = lds + (t & 1) * kBuf;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint4 b[QW][NS];
#pragma unroll
            for (int q = 0; q < QW; ++q)
#pragma unroll
                for (int h = 0; h < NS; ++h)
                    b[q][h] = *reinterpret_cast<const uint4 *>(
                        buf + ((ks * 4 + wq * QW + q) * NS + h) * 1024 +
                        (lane ^ ((((lane >> 4) & 1) << 1) | ((wq * QW + q) & 1))) * 16);
#pragma unroll
            for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
                for (int q = 0; q < QW; ++q) mfma_split<NS>(a[ks % AD][cb], b[q], acc[cb][q]);
            load_frags(s_begin + t * 4 + ks + AD, ks % AD);
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();
    }
#pragma unroll
    for (int q = 0; q < QW; ++q) {
        const int64_t j = j0 + (wq * QW + q) * 32 + (lane & 31);
        if (j >= n) continue;
#pragma unroll
        for (int cb = 0; cb < CBW; ++cb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int c = (wcb * CBW + cb) * 32 + d_row(v, lane);
                if (c < r) out[(int64_t)c * n + j] = NS == 1 ? acc[cb][q][v] * out_scale[c] : acc[cb][q][v];
            }
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static inline int ns_of(int mma) { return mma == DLCX_MMA_F32 ? 3 : 2; }
static inline int cb_of(int r) { return r <= 32 ? 1 : r <= 64 ? 2 : r <= 128 ? 4 : 8; }
static inline size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }

struct QPlan {
    int JB, S, depth;
    int64_t ksteps_per_wave, KS;
};

static QPlan q_plan(int64_t m, int64_t n, int r, int K) {
    QPlan p;
    const int cb = cb_of(r);
    // 128 columns per workgroup in both Q kernels
    p.JB = 4;
    p.depth = 2;                           // k-steps (16 rows) of delta in flight per wavefront
    const int64_t col_wgs = ceil_div(n, 32 * p.JB) * K;
    // workgroups that run at once: two per compute unit; one at 8 basis blocks, where the
    // two-role kernel fills a unit by itself
    const int64_t cap = cb == 8 ? 256 : 512;
    int64_t S = ceil_div(cap, col_wgs);
    const int64_t smax = ceil_div(m, 64 * p.depth * 2);  // at least 2 pipeline rounds per wave
    if (S > smax) S = smax;
    if (S < 1) S = 1;
    if (S > 64) S = 64;
    p.S = (int)S;
    int64_t kpw = ceil_div(ceil_div(m, 16), (int64_t)p.S * 4);
    p.ksteps_per_wave = ceil_div(kpw, p.depth) * p.depth;
    p.KS = p.ksteps_per_wave * 4 * p.S;
    return p;
}

// scratch of the fp16 form at the end of the fragment area: in_scale[256], out_scale[256], record
constexpr size_t kF16ScratchBytes = (2 * DLCX_MAX_RANK + 64) * sizeof(float);

size_t mfma_project_workspace_bytes(int mma, int64_t m, int64_t n, int r, int K) {
    // DLCX_MMA_F16: one fp16 piece beside the two bf16 pieces of the stand-by launch
    const int ns = mma == DLCX_MMA_F16 ? 3 : ns_of(mma), cb = cb_of(r);
    const size_t p_frags = (size_t)ceil_div(n, 64) * 4 * cb * ns * 1024;
    const QPlan q = q_plan(m, n, r, K);
    const size_t q_frags = (size_t)q.KS * cb * ns * 1024;
    const size_t slabs = q.S > 1 ? (size_t)K * q.S * r * n * sizeof(float) : 0;
    const size_t a = a256(p_frags), b = a256(q_frags) + a256(slabs);
    return (a > b ? a : b) + (mma == DLCX_MMA_F16 ? a256(kF16ScratchBytes) : 0);
}

template <int NS>
static int pack_kcontig(const float *src, int nrows, int64_t L, int RB, int64_t KS, uint4 *frags,
                        hipStream_t st, const float *row_scale = nullptr) {
    const int64_t nf = KS * RB;
    Timed timed(KID_PACK, st);
    hipLaunchKernelGGL(pack_kcontig_kernel<NS>, dim3((unsigned)ceil_div(nf, 4)), dim3(kW), 0, st,
                       src, nrows, L, RB, KS, frags, row_scale);
    return check_launch("pack_kcontig");
}

// scales and record of the fp16 form inside its scratch block
struct F16Scratch {
    float *in_scale, *out_scale;
    uint32_t *record;
};
static F16Scratch f16_scratch(void *block) {
    F16Scratch f;
    f.in_scale = reinterpret_cast<float *>(block);
    f.out_scale = f.in_scale + DLCX_MAX_RANK;
    f.record = reinterpret_cast<uint32_t *>(f.out_scale + DLCX_MAX_RANK);
    return f;
}
static int basis_scales(const float *basis, int r, int64_t L, const F16Scratch &f, hipStream_t st) {
    Timed timed(KID_PACK, st);
    hipLaunchKernelGGL(basis_scale_kernel, dim3((unsigned)r), dim3(kW), 0, st, basis, L, f.in_scale,
                       f.out_scale, f.record);
    return check_launch("basis_scale");
}

template <int NS, int CBW, int WC, int WK, int WR, int RB>
static int project_p_launch(const PtrPack<const float *> &delta, const uint4 *frags,
                            const PtrPack<float *> &out, int64_t m, int64_t n, int r, int K,
                            hipStream_t st) {
    constexpr int lds = project_p_lds_bytes<NS, CBW, WC, WK, WR, RB>();
    static size_t granted = 0;
    int rc = grant_dynamic_lds(
        reinterpret_cast<const void *>(project_p_mfma_kernel<NS, CBW, WC, WK, WR, RB>), lds,
        &granted, "project_p attribute");
    if (rc != DLCX_OK) return rc;
    const dim3 grid((unsigned)ceil_div(m, 32 * RB), (unsigned)K);
    hipLaunchKernelGGL((project_p_mfma_kernel<NS, CBW, WC, WK, WR, RB>), grid, dim3(kW), lds, st,
                       delta, frags, out, m, n, r);
    return DLCX_OK;
}

template <int NS, int CBW, int WC, int WR, int RB>
static int project_p_ws_launch(const PtrPack<const float *> &delta, const uint4 *frags,
                               const PtrPack<float *> &out, int64_t m, int64_t n, int r, int K,
                               hipStream_t st, uint32_t *record = nullptr,
                               const float *out_scale = nullptr, const uint32_t *guard = nullptr) {
    constexpr int lds = 2 * NS * 32 * RB * kPPitch;
    static size_t granted = 0;
    int rc = grant_dynamic_lds(
        reinterpret_cast<const void *>(project_p_ws_kernel<NS, CBW, WC, WR, RB>), lds, &granted,
        "project_p attribute");
    if (rc != DLCX_OK) return rc;
    const dim3 grid((unsigned)ceil_div(m, 32 * RB), (unsigned)K);
    hipLaunchKernelGGL((project_p_ws_kernel<NS, CBW, WC, WR, RB>), grid, dim3(kWs), lds, st, delta,
                       frags, out, m, n, r, record, out_scale, guard);
    return DLCX_OK;
}

// The projection at 4 or 8 basis blocks (ranks above 64) in its fp16 form, where the matrix cores
// and not the stream of delta set the pace: one fp16 product per block instead of three bf16
// ones, followed by the bf16 kernel as a stand-by that returns at once unless the fp16 launch
// recorded a largest |delta| outside the window in which fp16 is safe.  False: not applicable
// (fewer basis blocks, or too few rows for the two-role kernel), the caller goes on as usual.
static bool project_p_f16(int64_t m, int64_t n, int r, int K, const PtrPack<const float *> &delta,
                          const float *q_in, const PtrPack<float *> &out, void *workspace,
                          hipStream_t st, int *rc_out) {
    const int cb = cb_of(r);
    if (cb < 4 || ceil_div(m, 128) * K < 256) return false;
    const int64_t KS = ceil_div(n, 64) * 4;
    char *ws = reinterpret_cast<char *>(workspace);
    uint4 *frags2 = reinterpret_cast<uint4 *>(ws);                                // two bf16 pieces
    uint4 *frags1 = reinterpret_cast<uint4 *>(ws + (size_t)KS * cb * 2 * 1024);   // one fp16 piece
    const F16Scratch f = f16_scratch(ws + a256((size_t)KS * cb * 3 * 1024));
    int rc = basis_scales(q_in, r, n, f, st);
    if (rc == DLCX_OK) rc = pack_kcontig<1>(q_in, r, n, cb, KS, frags1, st, f.in_scale);
    if (rc == DLCX_OK) rc = pack_kcontig<2>(q_in, r, n, cb, KS, frags2, st);
    if (rc == DLCX_OK) {
        Timed timed(KID_PROJECT_P, st);
        if (cb == 4) {
            rc = project_p_ws_launch<1, 2, 2, 2, 4>(delta, frags1, out, m, n, r, K, st, f.record, f.out_scale);
            if (rc == DLCX_OK)
                rc = project_p_ws_launch<2, 2, 2, 2, 4>(delta, frags2, out, m, n, r, K, st, nullptr, nullptr, f.record);
        } else {
            rc = project_p_ws_launch<1, 2, 4, 1, 4>(delta, frags1, out, m, n, r, K, st, f.record, f.out_scale);
            if (rc == DLCX_OK)
                rc = project_p_ws_launch<2, 2, 4, 1, 4>(delta, frags2, out, m, n, r, K, st, nullptr, nullptr, f.record);
        }
        if (rc == DLCX_OK) rc = check_launch("project_p_f16");
    }
    *rc_out = rc;
    return true;
}

template <int NS>
static int project_p_ns(int64_t m, int64_t n, int r, int K, const PtrPack<const float *> &delta,
                        const float *q_in, const PtrPack<float *> &out, void *workspace,
                        hipStream_t st) {
    const int cb = cb_of(r);
    const int64_t KS = ceil_div(n, 64) * 4;
    uint4 *frags = reinterpret_cast<uint4 *>(workspace);
    int rc = pack_kcontig<NS>(q_in, r, n, cb, KS, frags, st);
    if (rc != DLCX_OK) return rc;
    Timed timed(KID_PROJECT_P, st);
    switch (cb) {
        case 1: rc = project_p_launch<NS, 1, 1, 2, 2, 2>(delta, frags, out, m, n, r, K, st); break;
        case 2:
            if (ceil_div(m, 128) * K >= 256)
                rc = project_p_ws_launch<NS, 1, 2, 2, 4>(delta, frags, out, m, n, r, K, st);
            else
                rc = project_p_launch<NS, 2, 1, 2, 2, 2>(delta, frags, out, m, n, r, K, st);
            break;
        case 4:
            if (ceil_div(m, 128) * K >= 256)
                rc = project_p_ws_launch<NS, 2, 2, 2, 4>(delta, frags, out, m, n, r, K, st);
            else
                rc = project_p_launch<NS, 2, 2, 1, 2, 2>(delta, frags, out, m, n, r, K, st);
            break;
        default:
            // 128 rows per workgroup once that still gives every compute unit a workgroup
            if (ceil_div(m, 128) * K >= 256)
                rc = project_p_ws_launch<NS, 2, 4, 1, 4>(delta, frags, out, m, n, r, K, st);
            else
                rc = project_p_launch<NS, 2, 4, 1, 1, 2>(delta, frags, out, m, n, r, K, st);
            break;
    }
    if (rc != DLCX_OK) return rc;
    return check_launch("project_p_mfma");
}

int launch_sum_slabs(int K, const PtrPack<const float *> &slabs, const PtrPack<float *> &outs,
                     int64_t count, int S, int64_t slab_stride, hipStream_t st);

template <int NS, int CBW, int WCB>
static int project_q_ws_launch(const dim3 &grid, hipStream_t st, const PtrPack<const float *> &delta,
                               const uint4 *frags, const PtrPack<float *> &dst, int64_t m,
                               int64_t n, int r, int64_t ksteps_per_wg, int64_t slab,
                               uint32_t *record = nullptr, const float *out_scale = nullptr,
                               const uint32_t *guard = nullptr) {
    constexpr int lds = 2 * 16 * NS * 1024;
    static size_t granted = 0;
    int rc = grant_dynamic_lds(reinterpret_cast<const void *>(project_q_ws_kernel<NS, CBW, WCB>),
                               lds, &granted, "project_q attribute");
    if (rc != DLCX_OK) return rc;
    hipLaunchKernelGGL((project_q_ws_kernel<NS, CBW, WCB>), grid, dim3(kWs), lds, st, delta, frags, dst,
                       m, n, r, ksteps_per_wg, slab, record, out_scale, guard);
    return DLCX_OK;
}

// F16: the fp16 form for 4 or 8 basis blocks (see project_p_f16), with the bf16 kernel as its
// stand-by; NS is then the stand-by's piece count (2) and the workspace holds three pieces.
template <int NS, bool F16>
static int project_q_ns(int64_t m, int64_t n, int r, int K, const PtrPack<const float *> &delta,
                        const float *p_hat, const PtrPack<float *> &out, void *workspace,
                        hipStream_t st) {
    const int cb = cb_of(r);
    const QPlan q = q_plan(m, n, r, K);
    const bool f16 = F16 && cb >= 4;
    const int pieces = F16 ? 3 : NS;  // as the workspace was sized
    char *wsb = reinterpret_cast<char *>(workspace);
    uint4 *frags = reinterpret_cast<uint4 *>(wsb);
    uint4 *frags1 = reinterpret_cast<uint4 *>(wsb + (size_t)q.KS * cb * NS * 1024);
    F16Scratch f = f16_scratch(nullptr);
    int rc = DLCX_OK;
    if (f16) {
        const size_t slab_bytes = q.S > 1 ? a256((size_t)K * q.S * r * n * sizeof(float)) : 0;
        f = f16_scratch(wsb + a256((size_t)q.KS * cb * pieces * 1024) + slab_bytes);
        rc = basis_scales(p_hat, r, m, f, st);
        if (rc == DLCX_OK) rc = pack_kcontig<1>(p_hat, r, m, cb, q.KS, frags1, st, f.in_scale);
        if (rc != DLCX_OK) return rc;
    }
    rc = pack_kcontig<NS>(p_hat, r, m, cb, q.KS, frags, st);
    if (rc != DLCX_OK) return rc;
    const int64_t slab = (int64_t)r * n;
    PtrPack<float *> dst = out;
    if (q.S > 1) {
        float *base = reinterpret_cast<float *>(wsb + a256((size_t)q.KS * cb * pieces * 1024));
        for (int k = 0; k < K; ++k) dst.p[k] = base + (int64_t)k * q.S * slab;
    }
    const dim3 grid((unsigned)ceil_div(n, 32 * q.JB), (unsigned)K, (unsigned)q.S);
    {
    Timed timed(KID_PROJECT_Q, st);
    if (f16) {  // the stand-by launches below then carry the record as their guard
        if (cb == 4) rc = project_q_ws_launch<1, 1, 4>(grid, st, delta, frags1, dst, m, n, r, q.ksteps_per_wave * 4, slab, f.record, f.out_scale);
        else rc = project_q_ws_launch<1, 2, 4>(grid, st, delta, frags1, dst, m, n, r, q.ksteps_per_wave * 4, slab, f.record, f.out_scale);
        if (rc != DLCX_OK) return rc;
    }
    const uint32_t *guard = f16 ? f.record : nullptr;
    switch (cb) {
        case 1: hipLaunchKernelGGL((project_q_mfma_kernel<NS, 1, 4, 2>), grid, dim3(kW), 0, st, delta, frags, dst, m, n, r, q.ksteps_per_wave, slab); break;
        case 2: rc = project_q_ws_launch<NS, 1, 2>(grid, st, delta, frags, dst, m, n, r, q.ksteps_per_wave * 4, slab); break;
        case 4: rc = project_q_ws_launch<NS, 1, 4>(grid, st, delta, frags, dst, m, n, r, q.ksteps_per_wave * 4, slab, nullptr, nullptr, guard); break;
        default: rc = project_q_ws_launch<NS, 2, 4>(grid, st, delta, frags, dst, m, n, r, q.ksteps_per_wave * 4, slab, nullptr, nullptr, guard); break;
    }
    if (rc == DLCX_OK) rc = check_launch("project_q_mfma");
    }
    if (rc != DLCX_OK || q.S == 1) return rc;
    PtrPack<const float *> src;
    for (int k = 0; k < K; ++k) src.p[k] = dst.p[k];
    return launch_sum_slabs(K, src, out, slab, q.S, slab, st);
}

int launch_project_p_mfma(int mma, int64_t m, int64_t n, int r, int K,
                          const PtrPack<const float *> &delta, const float *q_in,
                          const PtrPack<float *> &out, void *workspace, hipStream_t st) {
    if (mma == DLCX_MMA_F32) return project_p_ns<3>(m, n, r, K, delta, q_in, out, workspace, st);
    int rc = DLCX_OK;
    if (mma == DLCX_MMA_F16 && project_p_f16(m, n, r, K, delta, q_in, out, workspace, st, &rc))
        return rc;
    return project_p_ns<2>(m, n, r, K, delta, q_in, out, workspace, st);
}

int launch_project_q_mfma(int mma, int64_t m, int64_t n, int r, int K,
                          const PtrPack<const float *> &delta, const float *p_hat,
                          const PtrPack<float *> &out, void *workspace, hipStream_t st) {
    if (mma == DLCX_MMA_F32)
        return project_q_ns<3, false>(m, n, r, K, delta, p_hat, out, workspace, st);
    if (mma == DLCX_MMA_F16)
        return project_q_ns<2, true>(m, n, r, K, delta, p_hat, out, workspace, st);
    return project_q_ns<2, false>(m, n, r, K, delta, p_hat, out, workspace, st);
}

size_t mfma_reconstruct_workspace_bytes(int mma, int64_t m, int64_t n, int r) {
    const int ns = ns_of(mma);
    const size_t ks = (size_t)(r + 15) / 16;
    return a256((size_t)ceil_div(m, 32) * ks * ns * 1024) + a256((size_t)ceil_div(n, 32) * ks * ns * 1024);
}

template <int NS>
static int reconstruct_launch(int64_t m, int64_t n, int ks, const uint4 *pf, const uint4 *qf,
                              const ReconEpilogue &ep, hipStream_t st) {
    // Columns per workgroup: one 32 x 256 tile each, workgroups in tile order along the row block.
    // This kernel leaves no partial sums behind, so nothing speaks for longer column ranges, and
    // short ranges in tile order are what the memory system likes best (measured at rank 200:
    // 28672 x 8192 5.08 -> 5.63 TB/s against ranges of 1792 columns, 8192 x 28672 4.85 -> 5.12,
    // 8192 x 8192 5.2 -> 5.45; one or two long ranges per row block: 3.0 - 4.6).
    const int64_t rows = ceil_div(m, 32);
    const int64_t cols = 256;
    const dim3 grid((unsigned)ceil_div(n, cols), (unsigned)rows);
    Timed timed(KID_RECONSTRUCT, st);
    hipLaunchKernelGGL(reconstruct_mfma_kernel<NS>, grid, dim3(kW), 0, st, pf, qf, ep, m, n, cols,
                       ks);
    return check_launch("reconstruct_mfma");
}

template <int NS>
static int reconstruct_ns(int64_t m, int64_t n, int r, const float *p_hat, const float *q_bar,
                          const ReconEpilogue &ep, void *workspace, hipStream_t st) {
    const int ks = (r + 15) / 16;
    const int64_t xbm = ceil_div(m, 32), xbn = ceil_div(n, 32);
    uint4 *pf = reinterpret_cast<uint4 *>(workspace);
    uint4 *qf = reinterpret_cast<uint4 *>(reinterpret_cast<char *>(workspace) +
                                          a256((size_t)xbm * ks * NS * 1024));
    int rc;
    {
        Timed timed(KID_PACK, st);
        hipLaunchKernelGGL(pack_kstrided_kernel<NS>, dim3((unsigned)ceil_div(xbm * ks, 4)), dim3(kW), 0,
                           st, p_hat, r, m, ks, xbm, pf);
        rc = check_launch("pack p_hat");
    }
    if (rc != DLCX_OK) return rc;
    {
        Timed timed(KID_PACK, st);
        hipLaunchKernelGGL(pack_kstrided_kernel<NS>, dim3((unsigned)ceil_div(xbn * ks, 4)), dim3(kW), 0,
                           st, q_bar, r, n, ks, xbn, qf);
        rc = check_launch("pack q_bar");
    }
    if (rc != DLCX_OK) return rc;
    return reconstruct_launch<NS>(m, n, ks, pf, qf, ep, st);
}

int launch_reconstruct_mfma(int mma, int64_t m, int64_t n, int r, const float *p_hat,
                            const float *q_bar, const ReconEpilogue &ep, void *workspace,
                            hipStream_t st) {
    if (mma == DLCX_MMA_F32) return reconstruct_ns<3>(m, n, r, p_hat, q_bar, ep, workspace, st);
    return reconstruct_ns<2>(m, n, r, p_hat, q_bar, ep, workspace, st);
}

// ---- fused round: workspace layout and launch ------------------------------------------------
constexpr int kComputeUnits = 256;
struct RoundPlan {
    int chunks;        // column ranges per row block = slabs per worker
    int64_t cols;      // columns per workgroup (multiple of 256)
    int kc;            // workers per launch
};

static RoundPlan round_plan(int64_t m, int64_t n, int r) {
    RoundPlan p;
    (void)r;
    p.kc = 4;  // workers per launch: 4 x 2 basis blocks x 16 accumulator registers per wavefront
    // Column ranges per row block, from sweeps of this kernel over the benchmark shapes (one
    // workgroup occupies a compute unit): four ranges once the matrix is 2048 columns wide (at
    // 8192 columns 13 % faster than one or two, whatever the number of rows; at 28672 columns
    // the count does not matter), one for narrower matrices; more, up to eight, when that is
    // what it takes to give every compute unit two workgroups, but never ranges under 512
    // columns (two tiles per wavefront), where start-up and the slab sums cost more than a
    // fuller machine gains.
    const int64_t rows = ceil_div(m, 32);
    int64_t chunks = n >= 2048 ? 4 : 1;
    const int64_t need = ceil_div(2 * kComputeUnits, rows);
    if (chunks < need) chunks = need < 8 ? need : 8;
    const int64_t widest = n / 512 > 1 ? n / 512 : 1;
    if (chunks > widest) chunks = widest;
    p.cols = ceil_div(ceil_div(n, chunks), 256) * 256;
    p.chunks = (int)ceil_div(n, p.cols);
    return p;
}

// [basis fragments | P_hat_prev fragments | Q_bar_prev fragments | slabs (K x chunks x r x m)]
size_t mfma_round_workspace_bytes(int mma, int64_t m, int64_t n, int r, int r_prev, int K) {
    const int ns = ns_of(mma);
    const RoundPlan pl = round_plan(m, n, r);
    const size_t ksp = (size_t)(r_prev + 15) / 16;
    size_t total = a256((size_t)ceil_div(n, 64) * 4 * cb_of(r) * ns * 1024);
    total += a256((size_t)ceil_div(m, 32) * ksp * ns * 1024);
    total += a256((size_t)ceil_div(n, 32) * ksp * ns * 1024);
    if (pl.chunks > 1) total += a256((size_t)K * pl.chunks * r * m * sizeof(float));
    return total;
}

template <int NS, int CB, int KC, bool TLBF16>
static int round_launch_t(const uint4 *pf, const uint4 *qf, int ks, const uint4 *bf,
                        const ReconEpilogue &ep, const PtrPack<float *> &pslab, int64_t m,
                        int64_t n, int r, const RoundPlan &pl, int64_t slab_stride,
                        hipStream_t st) {
    const size_t basis = (NS == 2 && CB <= 2) ? (size_t)4 * CB * NS * 1024 : 0;
    const size_t tiles = 4 * (32 * kRPitch * 4) + 4 * (size_t)(NS * 32 * kPPitch) + 4 * basis;
    const size_t red = (size_t)KC * CB * 16 * 64 * 4;
    const size_t lds = tiles > red ? tiles : red;
    static size_t granted = 0;
    int rc = grant_dynamic_lds(reinterpret_cast<const void *>(round_mfma_kernel<NS, CB, KC, TLBF16>),
                               lds, &granted, "round kernel attribute");
    if (rc != DLCX_OK) return rc;
    const dim3 grid((unsigned)pl.chunks, (unsigned)ceil_div(m, 32));
    Timed timed(KID_ROUND, st);
    hipLaunchKernelGGL((round_mfma_kernel<NS, CB, KC, TLBF16>), grid, dim3(kW), lds, st, pf, qf, ks,
                       bf, ep, pslab, m, n, r, pl.cols, slab_stride);
    return check_launch("round_mfma");
}

template <int NS, int CB, int KC>
static int round_launch(const uint4 *pf, const uint4 *qf, int ks, const uint4 *bf,
                        const ReconEpilogue &ep, const PtrPack<float *> &pslab, int64_t m,
                        int64_t n, int r, const RoundPlan &pl, int64_t slab_stride,
                        hipStream_t st) {
    if (ep.tl_bf16)
        return round_launch_t<NS, CB, KC, true>(pf, qf, ks, bf, ep, pslab, m, n, r, pl, slab_stride, st);
    return round_launch_t<NS, CB, KC, false>(pf, qf, ks, bf, ep, pslab, m, n, r, pl, slab_stride, st);
}

template <int NS>
static int round_ns(int64_t m, int64_t n, int r, int r_prev, const float *p_hat, const float *q_bar,
                    const float *basis, const ReconEpilogue &ep_all, const PtrPack<float *> &factors,
                    void *workspace, hipStream_t st) {
    const int cb = cb_of(r);
    const RoundPlan pl = round_plan(m, n, r);
    const int ks = (r_prev + 15) / 16;
    const int64_t xbm = ceil_div(m, 32), xbn = ceil_div(n, 32);
    char *ws = reinterpret_cast<char *>(workspace);
    uint4 *bf = reinterpret_cast<uint4 *>(ws);
    ws += a256((size_t)ceil_div(n, 64) * 4 * cb * NS * 1024);
    uint4 *pf = reinterpret_cast<uint4 *>(ws);
    ws += a256((size_t)xbm * ks * NS * 1024);
    uint4 *qf = reinterpret_cast<uint4 *>(ws);
    ws += a256((size_t)xbn * ks * NS * 1024);
    float *slabs = reinterpret_cast<float *>(ws);
    int rc = pack_kcontig<NS>(basis, r, n, cb, ceil_div(n, 64) * 4, bf, st);
    if (rc != DLCX_OK) return rc;
    if (ks > 0) {
        {
            Timed timed(KID_PACK, st);
            hipLaunchKernelGGL(pack_kstrided_kernel<NS>, dim3((unsigned)ceil_div(xbm * ks, 4)),
                               dim3(kW), 0, st, p_hat, r_prev, m, ks, xbm, pf);
            rc = check_launch("pack p_hat");
        }
        if (rc != DLCX_OK) return rc;
        {
            Timed timed(KID_PACK, st);
            hipLaunchKernelGGL(pack_kstrided_kernel<NS>, dim3((unsigned)ceil_div(xbn * ks, 4)),
                               dim3(kW), 0, st, q_bar, r_prev, n, ks, xbn, qf);
            rc = check_launch("pack q_bar");
        }
        if (rc != DLCX_OK) return rc;
    }
    const int64_t slab = (int64_t)r * m;
    for (int k0 = 0; k0 < ep_all.K; k0 += pl.kc) {
        ReconEpilogue ep = ep_all;
        ep.K = ep_all.K - k0 < pl.kc ? ep_all.K - k0 : pl.kc;
        ep.apply = ep_all.apply && (k0 + pl.kc >= ep_all.K);  // theta moves with the last group
        PtrPack<float *> dst;
        for (int k = 0; k < ep.K; ++k) {
            ep.ef.p[k] = ep_all.ef.p[k0 + k];
            ep.tl.p[k] = ep_all.tl.p[k0 + k];
            dst.p[k] = pl.chunks > 1 ? slabs + (int64_t)(k0 + k) * pl.chunks * slab
                                     : factors.p[k0 + k];
        }
        switch (cb) {  // ranks above 64 do not come here: see dlcx_ef_delta_apply_compress
            case 1: rc = round_launch<NS, 1, 4>(pf, qf, ks, bf, ep, dst, m, n, r, pl, slab, st); break;
            case 2: rc = round_launch<NS, 2, 4>(pf, qf, ks, bf, ep, dst, m, n, r, pl, slab, st); break;
            default: rc = DLCX_EINVAL; break;
        }
        if (rc != DLCX_OK) return rc;
    }
    if (pl.chunks == 1) return DLCX_OK;
    PtrPack<const float *> src;
    for (int k = 0; k < ep_all.K; ++k) src.p[k] = slabs + (int64_t)k * pl.chunks * slab;
    return launch_sum_slabs(ep_all.K, src, factors, slab, pl.chunks, slab, st);
}

int launch_round_mfma(int mma, int64_t m, int64_t n, int r, int r_prev, const float *p_hat,
                      const float *q_bar, const float *basis, const ReconEpilogue &ep,
                      const PtrPack<float *> &factors, void *workspace, hipStream_t st) {
    if (mma == DLCX_MMA_F32)
        return round_ns<3>(m, n, r, r_prev, p_hat, q_bar, basis, ep, factors, workspace, st);
    return round_ns<2>(m, n, r, r_prev, p_hat, q_bar, basis, ep, factors, workspace, st);
}

}  // namespace dlcx
