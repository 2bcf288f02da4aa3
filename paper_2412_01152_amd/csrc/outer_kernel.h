// Outer optimiser step (Algorithm 1, outer-optimisation line): SGD with Nesterov momentum,
//   m' = beta m + g,   theta' = theta - lr (g + beta m'),
// one streaming pass, in place, with g either an fp32 array or codes decoded through the
// segment's codebook (kept in LDS).  Optionally also writes theta' as the workers' new weights.
#pragma once

#include "device_common.h"

namespace diloco {

enum OutKind { kOutNone = 0, kOutF32 = 1, kOutBf16 = 2 };

// The caller loads m and theta for all unrolled positions before the first store: the arrays are
// updated in place, so the compiler cannot move a later load above an earlier store by itself.
template <int kOut>
__device__ __forceinline__ void nesterov4(float* theta, float* mom, void* local_out, uint64_t i,
                                          f32x4 g, f32x4 m, f32x4 th, float lr, float beta) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        m[e] = __fmaf_rn(beta, m[e], g[e]);
        th[e] = __fmaf_rn(-lr, __fmaf_rn(beta, m[e], g[e]), th[e]);
    }
    st_f32x4(mom + i, m);
    st_f32x4(theta + i, th);
    if (kOut == kOutF32) st_f32x4((float*)local_out + i, th);
    if (kOut == kOutBf16) {
        u16x4_u h;
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = f32_to_bf16_bits(th[e]);
        *(u16x4_u*)((uint16_t*)local_out + i) = h;
    }
}

template <int kOut>
__device__ __forceinline__ void nesterov1(float* theta, float* mom, void* local_out, uint64_t i,
                                          float g, float lr, float beta) {
    float m = __fmaf_rn(beta, mom[i], g);
    float th = __fmaf_rn(-lr, __fmaf_rn(beta, m, g), theta[i]);
    mom[i] = m;
    theta[i] = th;
    if (kOut == kOutF32) ((float*)local_out)[i] = th;
    if (kOut == kOutBf16) ((uint16_t*)local_out)[i] = f32_to_bf16_bits(th);
}

template <int kOut>
__global__ __launch_bounds__(kThreads) void outer_fp32_kernel(float* theta, float* mom,
                                                             const float* __restrict__ delta,
                                                             uint64_t N, Work work, float lr,
                                                             float beta, void* local_out) {
    __shared__ unsigned long long s_claim;
    const int tid = threadIdx.x;
    Claimer claimer(work);
    Share sh;
    const uint32_t phase = work.phase;
    while (claimer.claim(work, N, sh, &s_claim)) {
    uint64_t base = aligned_start(sh.begin, sh.end, phase);
    for (uint64_t i = sh.begin + tid; i < base; i += kThreads)
        nesterov1<kOut>(theta, mom, local_out, i, delta[i], lr, beta);
    for (; base + kIter <= sh.end; base += kIter) {
        f32x4 g[kUnroll], m[kUnroll], th[kUnroll];
#pragma unroll
        for (int j = 0; j < kUnroll; ++j) {
            const uint64_t i = base + (uint64_t)(j * kThreads + tid) * kVec;
            g[j] = ld_f32x4(delta + i);
            m[j] = ld_f32x4(mom + i);
            th[j] = ld_f32x4(theta + i);
        }
#pragma unroll
        for (int j = 0; j < kUnroll; ++j)
            nesterov4<kOut>(theta, mom, local_out, base + (uint64_t)(j * kThreads + tid) * kVec, g[j],
                            m[j], th[j], lr, beta);
    }
    for (uint64_t i = base + tid; i < sh.end; i += kThreads)
        nesterov1<kOut>(theta, mom, local_out, i, delta[i], lr, beta);
    }
}

template <int kOut>
__global__ __launch_bounds__(kThreads) void outer_coded_kernel(float* theta, float* mom,
                                                              const uint8_t* __restrict__ codes,
                                                              const float* __restrict__ lut,
                                                              const uint64_t* __restrict__ seg,
                                                              uint32_t T, uint64_t N,
                                                              Work work, float lr, float beta,
                                                              void* local_out) {
    __shared__ float s_lut[kBuckets];
    __shared__ unsigned long long s_claim;
    const int tid = threadIdx.x;
    Claimer claimer(work);
    Share sh;
    while (claimer.claim(work, N, sh, &s_claim)) {
    uint32_t s = find_segment(seg, T, sh.begin);
    uint64_t pos = sh.begin;
    while (pos < sh.end) {
        const uint64_t seg_end = seg[s + 1];
        if (seg_end <= pos) {
            ++s;
            continue;
        }
        const uint64_t sub_end = seg_end < sh.end ? seg_end : sh.end;
        __syncthreads();
        s_lut[tid] = lut[(size_t)s * kBuckets + tid];
        __syncthreads();
        uint64_t base = aligned_start(pos, sub_end, work.phase);
        for (uint64_t i = pos + tid; i < base; i += kThreads)
            nesterov1<kOut>(theta, mom, local_out, i, s_lut[codes[i]], lr, beta);
        for (; base + kIter <= sub_end; base += kIter) {
            uint32_t c[kUnroll];
            f32x4 m[kUnroll], th[kUnroll];
#pragma unroll
            for (int j = 0; j < kUnroll; ++j) {
                const uint64_t i = base + (uint64_t)(j * kThreads + tid) * kVec;
                c[j] = ld_u8x4(codes + i);
                m[j] = ld_f32x4(mom + i);
                th[j] = ld_f32x4(theta + i);
            }
#pragma unroll
            for (int j = 0; j < kUnroll; ++j) {
                f32x4 g;
#pragma unroll
                for (int e = 0; e < 4; ++e) g[e] = s_lut[(c[j] >> (8 * e)) & 0xffu];
                nesterov4<kOut>(theta, mom, local_out, base + (uint64_t)(j * kThreads + tid) * kVec, g,
                                m[j], th[j], lr, beta);
            }
        }
        for (uint64_t i = base + tid; i < sub_end; i += kThreads)
            nesterov1<kOut>(theta, mom, local_out, i, s_lut[codes[i]], lr, beta);
        pos = sub_end;
    }
    }
}

}  // namespace diloco
