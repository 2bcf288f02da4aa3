// Kernel templates of the quantising passes.
//
// Section 2.2's quantiser needs the statistics of a whole segment before any element can be coded,
// so every quantising call is two streaming passes over its input:
//   pass A  (stats_kernel)  values -> per-segment sum and sum of squares about a pivot, in fp64
//   pass B  (quant_kernel)  values -> bucket index per element + per-bucket {count, offset sum}
// with two tiny kernels between and after them that turn the sums into (lo, 1/width) and into the
// codebook.  "Values" come from a source functor: the pseudo-gradient theta_outer - theta_local
// (stage 1), the averaged fp32 sum of decoded peer contributions (stage 2), or a stored fp32 array.
// Nothing but codes, codebooks and (when asked for) the fp32 accumulation is written.
#pragma once

#include "device_common.h"

namespace diloco {

// ------------------------------------------------------------------------------------------
// sources
// ------------------------------------------------------------------------------------------

// Algorithm 1, outer-gradient line: d = theta_outer - theta_local, one fp32 subtraction.
template <bool kLocalBf16>
struct SrcPseudoGrad {
    const float* theta_outer;
    const void* theta_local;
    static constexpr int kLdsFloats = 0;
    static constexpr int kStage = kStageIters;      // pass B holds its codes back for the write window
    static constexpr int kQuantWaves = 1;           // pass B: no register budget asked for
    struct Raw {
        f32x4 a, b;
    };
    __device__ __forceinline__ void bind(float*) {}
    __device__ __forceinline__ void enter_segment(uint32_t) {}
    __device__ __forceinline__ Raw fetch4(uint64_t i) const {
        Raw r;
        r.a = ld_f32x4(theta_outer + i);
        if (kLocalBf16)
            r.b = ld_bf16x4((const uint16_t*)theta_local + i);
        else
            r.b = ld_f32x4((const float*)theta_local + i);
        return r;
    }
    __device__ __forceinline__ f32x4 value4(const Raw& r) const {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __fsub_rn(r.a[e], r.b[e]);
        return v;
    }
    __device__ __forceinline__ float value1(uint64_t i) const {
        float b = kLocalBf16 ? bf16_bits_to_f32(((const uint16_t*)theta_local)[i])
                             : ((const float*)theta_local)[i];
        return __fsub_rn(theta_outer[i], b);
    }
    __device__ __forceinline__ float sample_value(uint64_t i, uint32_t) const { return value1(i); }
};

// A stored fp32 array (second pass of stage 2 when the accumulation was written out).
struct SrcF32 {
    const float* x;
    static constexpr int kLdsFloats = 0;
    static constexpr int kStage = 0;                // staging gains nothing for a single read stream
    static constexpr int kQuantWaves = 1;
    struct Raw {
        f32x4 a;
    };
    __device__ __forceinline__ void bind(float*) {}
    __device__ __forceinline__ void enter_segment(uint32_t) {}
    __device__ __forceinline__ Raw fetch4(uint64_t i) const {
        Raw r;
        r.a = ld_f32x4(x + i);
        return r;
    }
    __device__ __forceinline__ f32x4 value4(const Raw& r) const { return r.a; }
    __device__ __forceinline__ float value1(uint64_t i) const { return x[i]; }
    __device__ __forceinline__ float sample_value(uint64_t i, uint32_t) const { return x[i]; }
};

// Section 2.2's reduction: decode each of the W coded contributions through its segment's
// codebook (held in LDS), add them in contribution order in fp32 on top of the optional
// un-quantised local value, then take the average of Algorithm 1 (division by k).
// The average is a compile-time choice between two forms: multiplication by `div` (used when the
// divisor is a power of two, 1 included: the product rounds exactly like the quotient) and a true
// correctly rounded fp32 division by `div`.
template <int W, bool kHasLocal, bool kTrueDiv>
struct SrcReduce {
    static constexpr int kW = W > 0 ? W : 1;
    const uint8_t* codes[kW];
    const float* luts[kW];     // each [T][256]
    const float* local;        // [n] or nullptr
    float div;                 // the divisor (kTrueDiv) or its exact reciprocal
    float* lds;                // W tables of 256 floats
    static constexpr int kLdsFloats = W * kBuckets;
    static constexpr int kStage = 0;                // the LDS goes to the bin copies and the tables
    // Pass B at W <= 4 is held to 128 registers, so that four blocks (which is what its LDS admits)
    // are resident per CU instead of three.
    static constexpr int kQuantWaves = W <= 4 ? 4 : 1;
    struct Raw {
        uint32_t c[kW];
        f32x4 l;
    };
    __device__ __forceinline__ void bind(float* p) { lds = p; }
    __device__ __forceinline__ void enter_segment(uint32_t s) {
        if (W > 0) {
            __syncthreads();
#pragma unroll
            for (int p = 0; p < W; ++p) {
                const float entry = luts[p][(size_t)s * kBuckets + threadIdx.x];
                // the sum starts from 0.0f: with no local addend its first addition (which only turns
                // -0 into +0) is done here, once per table entry, instead of once per element
                lds[p * kBuckets + threadIdx.x] = (p == 0 && !kHasLocal) ? __fadd_rn(0.0f, entry) : entry;
            }
            __syncthreads();
        }
    }
    __device__ __forceinline__ float finish(float v) const {
        return kTrueDiv ? __fdiv_rn(v, div) : __fmul_rn(v, div);
    }
    __device__ __forceinline__ Raw fetch4(uint64_t i) const {
        Raw r;
#pragma unroll
        for (int p = 0; p < W; ++p) r.c[p] = ld_u8x4(codes[p] + i);
        if (kHasLocal) r.l = ld_f32x4(local + i);
        return r;
    }
    __device__ __forceinline__ f32x4 value4(const Raw& r) const {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float acc = kHasLocal ? r.l[e] : 0.0f;
#pragma unroll
            for (int p = 0; p < W; ++p) {
                const float x = lds[p * kBuckets + ((r.c[p] >> (8 * e)) & 0xffu)];
                acc = (p == 0 && !kHasLocal) ? x : __fadd_rn(acc, x);
            }
            v[e] = finish(acc);
        }
        return v;
    }
    __device__ __forceinline__ float value1(uint64_t i) const {
        float acc = kHasLocal ? local[i] : 0.0f;
#pragma unroll
        for (int p = 0; p < W; ++p) {
            const float x = lds[p * kBuckets + codes[p][i]];
            acc = (p == 0 && !kHasLocal) ? x : __fadd_rn(acc, x);
        }
        return finish(acc);
    }
    // Same value straight from global memory (no LDS tables needed): used for the pivot samples.
    __device__ __forceinline__ float sample_value(uint64_t i, uint32_t s) const {
        float acc = kHasLocal ? local[i] : 0.0f;
#pragma unroll
        for (int p = 0; p < W; ++p)
            acc = __fadd_rn(acc, luts[p][(size_t)s * kBuckets + codes[p][i]]);
        return finish(acc);
    }
};

// ------------------------------------------------------------------------------------------
// pass A: statistics (Section 2.2 item 1)
// ------------------------------------------------------------------------------------------
// Each thread keeps fp64 sums of (x - c) and (x - c)^2 about a pivot c that lies inside the bulk of
// the segment: the shift removes the cancellation of a large mean and makes a constant segment give
// exactly 0.  The variance is formed as (S2 - S1^2 / n) / (n - 1), which loses about (D / sigma)^2
// of fp64 precision when the pivot sits D away from the mean, so the pivot must not be an outlier:
// it is the median of nine values taken at evenly spread positions of the segment (first, 1/8, ...,
// last).  For the median to be an outlier at least five of the nine samples would have to be, and
// values that frequent dominate sigma themselves, so D / sigma stays small either way.
// The pivots are written by a one-thread-per-segment kernel before the pass starts, because the
// pass may overwrite its own input (accumulation stored in place over the local addend).
// One pair of fp64 atomics per (block, segment).  When kWriteAcc, the values are also stored.
constexpr int kPivotSamples = 9;
constexpr int kPivotLanes = 16;                      // lanes per segment (the first nine take a sample each)
constexpr int kPivotSegmentsPerBlock = kThreads / kPivotLanes;
template <class Src>
__global__ __launch_bounds__(kThreads) void pivot_kernel(Src src, const uint64_t* __restrict__ seg, uint32_t T,
                                                        float* __restrict__ pivot) {
    const uint32_t s = blockIdx.x * kPivotSegmentsPerBlock + threadIdx.x / kPivotLanes;
    const int j = threadIdx.x % kPivotLanes;
    uint64_t a = 0, n = 0;
    if (s < T) {
        a = seg[s];
        n = seg[s + 1] - a;
    }
    float mine = 0.0f;
    if (n > 0 && j < kPivotSamples) mine = src.sample_value(a + (uint64_t)j * (n - 1) / (kPivotSamples - 1), s);
    float v[kPivotSamples];
#pragma unroll
    for (int i = 0; i < kPivotSamples; ++i) v[i] = __shfl(mine, i, kPivotLanes);
    // odd-even transposition sort, fully unrolled (a NaN sample drops out: fminf / fmaxf return the
    // other operand; the statistics pass itself still sees it and the segment is flagged)
#pragma unroll
    for (int round = 0; round < kPivotSamples; ++round) {
#pragma unroll
        for (int i = round & 1; i + 1 < kPivotSamples; i += 2) {
            const float lo = fminf(v[i], v[i + 1]), hi = fmaxf(v[i], v[i + 1]);
            v[i] = lo;
            v[i + 1] = hi;
        }
    }
    if (s < T && j == 0) pivot[s] = n > 0 ? v[kPivotSamples / 2] : 0.0f;
}

template <class Src, bool kWriteAcc>
__global__ __launch_bounds__(kThreads) void stats_kernel(Src src_in, const uint64_t* __restrict__ seg,
                                                        uint32_t T, uint64_t N, Work work,
                                                        double* __restrict__ stats,
                                                        const float* __restrict__ pivot,
                                                        float* acc_out) {
    __shared__ float s_src[Src::kLdsFloats > 0 ? Src::kLdsFloats : 1];
    __shared__ double s_red[8];
    __shared__ unsigned long long s_claim;
    Src src = src_in;
    src.bind(s_src);
    const int tid = threadIdx.x;
    const uint32_t phase = work.phase;
    // Sums stay in registers across the block's chunks for as long as the segment stays the same;
    // they go to the segment's global accumulators when the segment changes and when the block
    // leaves.  (With one quantisation group per ring chunk every block would otherwise send one
    // pair of atomics per claim to the same two addresses.)
    uint32_t cur = kNoSegment;
    double c64 = 0.0, s1 = 0.0, s2 = 0.0;
    auto flush_segment = [&]() {                 // block-uniform
        block_sum2(s1, s2, s_red);
        if (tid == 0) {
            atomicAdd(&stats[2 * (size_t)cur], s1);
            atomicAdd(&stats[2 * (size_t)cur + 1], s2);
        }
        s1 = 0.0;
        s2 = 0.0;
    };
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
            if (s != cur) {
                if (cur != kNoSegment) flush_segment();
                cur = s;
                src.enter_segment(s);
                c64 = (double)pivot[s];
            }
            auto single = [&](uint64_t lo, uint64_t hi) {
                for (uint64_t i = lo + tid; i < hi; i += kThreads) {
                    float v = src.value1(i);
                    if (kWriteAcc) acc_out[i] = v;
                    double d = (double)v - c64;
                    s1 += d;
                    s2 = fma(d, d, s2);
                }
            };
            uint64_t base = aligned_start(pos, sub_end, phase);
            single(pos, base);
            for (; base + kIter <= sub_end; base += kIter) {
                typename Src::Raw raw[kUnroll];
#pragma unroll
                for (int j = 0; j < kUnroll; ++j)
                    raw[j] = src.fetch4(base + (uint64_t)(j * kThreads + tid) * kVec);
#pragma unroll
                for (int j = 0; j < kUnroll; ++j) {
                    f32x4 v = src.value4(raw[j]);
                    if (kWriteAcc) st_f32x4(acc_out + base + (uint64_t)(j * kThreads + tid) * kVec, v);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        double d = (double)v[e] - c64;
                        s1 += d;
                        s2 = fma(d, d, s2);
                    }
                }
            }
            single(base, sub_end);
            pos = sub_end;
        }
    }
    if (cur != kNoSegment) flush_segment();
}

// ------------------------------------------------------------------------------------------
// pass B: bucket index per element, and the per-bucket sums behind the codebook (item 4)
// ------------------------------------------------------------------------------------------
// The codebook needs, per bucket, the count and the sum of the values in it.  Floating-point LDS
// atomics are several times slower than integer ones on this chip, so the sum is kept in fixed
// point: for a value x in bucket k the kernel forms off = x - centre_k (|off| <= half a bucket),
// lets fma(off, 2^21 / width, 1.5 * 2^23) round it to an integer q in the low mantissa bits, and
// adds the single 64-bit word  (1 << 48) | bits(that float)  to the bucket's LDS bin: count in the
// top 16 bits, sum of (0x4B400000 + q) in the low 48.  One rounding of at most 2^-22 of a bucket
// per element, integer sums exact and order-independent thereafter.
// Values further than one bucket width from their bucket's centre (the clipped tails that land in
// buckets 0 and 255) do not fit that format; they are rare and go through per-thread fp64
// accumulators instead.  Thread k owns bin k: every kFlushIters iterations (before either field can
// overflow) it moves the bin into 64-bit registers, and when the block leaves the segment it
// adds its totals to the segment's global integer bins.
// When the source is the reduce, this pass keeps the vector ALUs and the LDS about as busy as the
// memory (about 22 vector instructions per element at W = 4), so the per-element chain is kept
// short: no mask on the index, no mask on the addend, the half bucket folded into centre_0.
struct PassBOut {
    unsigned long long* hsumq;   // [T][256] signed sum of q (two's complement)
    unsigned long long* hcnt;    // [T][256]
    double* osum;                // [T][2]   fp64 sum of off of the far values in bucket 0 / 255
    unsigned long long* ocnt;    // [T][2]
};

struct BinScale {
    float lo, inv_w, w, centre0, scale, reach;
};
__device__ __forceinline__ BinScale bin_scale(float lo, float inv_w) {
    BinScale b;
    b.lo = lo;
    b.inv_w = inv_w;
    b.w = bucket_width(inv_w);
    b.centre0 = bucket_centre0(lo, b.w);
    b.scale = offset_scale(inv_w);
    b.reach = b.scale > 0.0f ? b.w : 0.0f;   // no fixed-point scale: only exact zeros take the fast path
    return b;
}

struct FarSums {
    double lo_sum = 0.0, hi_sum = 0.0;
    unsigned lo_cnt = 0, hi_cnt = 0;
};

__device__ __forceinline__ void far_add(float off, int k, FarSums& far) {
    if (k == 0) {              // a value below the range is clipped into bucket 0, everything else
        far.lo_sum += (double)off;   // that is far from its centre sits in bucket 255
        far.lo_cnt += 1;
    } else {
        far.hi_sum += (double)off;
        far.hi_cnt += 1;
    }
}

// The float holding round(off * scale) in its low mantissa bits; its bit pattern is the bin addend.
__device__ __forceinline__ unsigned long long bin_addend(float off, float scale) {
    return (1ull << kCountShift) | (unsigned long long)__float_as_uint(__fmaf_rn(off, scale, kRoundMagic));
}

// The bucket index comes out of a clamp to [0, 255] (NaN gives 0), so its conversion needs no mask.
__device__ __forceinline__ int code_and_bin(float x, const BinScale& b, unsigned long long* s_bin,
                                            int copies, FarSums& far) {
    const float kf = bucket_of_f(x, b.lo, b.inv_w);
    const int k = (int)(unsigned)kf;
    const float off = __fsub_rn(x, bucket_centre(kf, b.centre0, b.w));
    if (fabsf(off) <= b.reach)
        atomicAdd(&s_bin[k * copies], bin_addend(off, b.scale));
    else
        far_add(off, k, far);
    return k;
}

// Four values at once: the four index / offset chains are independent, the bin updates are
// predicated, and the rare far values of the group are handled behind a single branch.
__device__ __forceinline__ uint32_t code_and_bin4(f32x4 v, const BinScale& b, unsigned long long* s_bin,
                                                  int copies, FarSums& far) {
    int k[4];
    float off[4];
    bool near[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float kf = bucket_of_f(v[e], b.lo, b.inv_w);
        k[e] = (int)(unsigned)kf;
        off[e] = __fsub_rn(v[e], bucket_centre(kf, b.centre0, b.w));
        near[e] = fabsf(off[e]) <= b.reach;
        if (near[e]) atomicAdd(&s_bin[k[e] * copies], bin_addend(off[e], b.scale));
    }
    if (!(near[0] & near[1] & near[2] & near[3])) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (!near[e]) far_add(off[e], k[e], far);
    }
    return (uint32_t)k[0] | ((uint32_t)k[1] << 8) | ((uint32_t)k[2] << 16) | ((uint32_t)k[3] << 24);
}

// The bucket indices alone, for a codebook that needs no bucket sums (bucket midpoints).
__device__ __forceinline__ int code_only(float x, const BinScale& b) {
    return (int)(unsigned)bucket_of_f(x, b.lo, b.inv_w);
}
__device__ __forceinline__ uint32_t code_only4(f32x4 v, const BinScale& b) {
    uint32_t k[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) k[e] = (uint32_t)bucket_of_f(v[e], b.lo, b.inv_w);
    return k[0] | (k[1] << 8) | (k[2] << 16) | (k[3] << 24);
}

// kCopies: each bucket's LDS bin exists kCopies times, copy (lane mod kCopies) at consecutive
// addresses, so that neighbouring lanes hit different banks even when they hit the same bucket
// (a 64-bit bin spans two of the 32 banks; with 16 copies 16 consecutive lanes never collide).
// kCopies == 0: no bins at all - the pass only writes codes (the midpoint codebook of the quantiser
// variants is a function of the range alone), which takes the LDS atomics, the offset arithmetic and
// the flushes out of the loop.
//
// Writing the codes.  On this chip a steady trickle of writes next to the read streams costs far
// more than its bytes.  The codes of whole iterations are therefore kept in LDS (kStage iterations
// of 4 KiB) and written out only inside a short window that recurs with a fixed period of the
// chip-wide constant-rate clock, the same window for every block, or when the staging area is
// full: HBM then sees long read phases and short write phases.  Nobody waits for anybody: a block
// looks at the clock after each iteration and carries on.  Sources whose pass B needs its LDS for
// other things, or gains nothing, set kStage = 0.
template <class Src, int kCopies, int kStage>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(Src::kQuantWaves))) void quant_kernel(Src src_in, const uint64_t* __restrict__ seg,
                                                        uint32_t T, uint64_t N, Work work,
                                                        const diloco_qparams* __restrict__ qp,
                                                        uint8_t* __restrict__ codes, PassBOut out,
                                                        WritePhase phase_cfg) {
    __shared__ float s_src[Src::kLdsFloats > 0 ? Src::kLdsFloats : 1];
    constexpr bool kBins = kCopies > 0;
    __shared__ unsigned long long s_bin_all[kBins ? kBuckets * kCopies : 1];
    __shared__ double s_red[8];
    __shared__ unsigned long long s_claim;
    // staged codes and the element index each staged iteration starts at (kStage == 0: no staging)
    __shared__ __attribute__((aligned(16))) uint32_t s_stage[kStage > 0 ? kStage * (kIter / 4) : 4];
    __shared__ uint64_t s_stage_at[kStage > 0 ? kStage : 1];
    const bool phased = kStage > 0 && phase_cfg.period != 0;
    Src src = src_in;
    src.bind(s_src);
    const int tid = threadIdx.x;
    unsigned long long* const s_bin = s_bin_all + (kBins ? (tid & (kCopies - 1)) : 0);   // this lane's copy
    const uint32_t phase = work.phase;
    // Bins and totals live across the block's chunks for as long as the segment stays the same: the
    // LDS bins are drained into registers before either of their fields can overflow, and the registers
    // go to the segment's global bins when the segment changes and when the block leaves.
    uint32_t cur = kNoSegment;
    BinScale bs = bin_scale(0.0f, 0.0f);
    long long bin_q = 0;
    unsigned long long bin_c = 0;
    FarSums far;
    uint32_t pending = 0;                        // elements binned since the last drain (block-uniform)
    constexpr uint32_t kDrainAfter = (uint32_t)kFlushIters * kIter;
    int staged = 0;                              // iterations whose codes sit in s_stage (block-uniform)
    auto write_staged = [&]() {                  // block-uniform; barrier before and after
        __syncthreads();
        for (int it = 0; it < staged; ++it) {
            const u32x4 v = *(const u32x4*)&s_stage[it * (kIter / 4) + tid * 4];
            st_u8x16(codes + s_stage_at[it] + (uint64_t)tid * 16, v);
        }
        __syncthreads();
        staged = 0;
    };
    if constexpr (kBins) {
#pragma unroll
        for (int c = 0; c < kCopies; ++c) s_bin_all[c * kBuckets + tid] = 0;
        __syncthreads();
    }
    // thread k sums and clears the kCopies copies of bin k, starting at a rotated copy so that the
    // lanes of a wave read different banks; callers put a barrier before and after
    auto drain = [&]() {
#pragma unroll
        for (int i = 0; i < (kBins ? kCopies : 0); ++i) {
            const int idx = tid * kCopies + ((i + tid) & (kCopies - 1));
            const unsigned long long packed = s_bin_all[idx];
            s_bin_all[idx] = 0;
            const unsigned long long c = packed >> kCountShift;
            bin_q += (long long)(packed & ((1ull << kCountShift) - 1)) - (long long)c * kAddendBase;
            bin_c += c;
        }
        pending = 0;
    };
    auto flush_segment = [&]() {                 // block-uniform
        if constexpr (!kBins) return;
        __syncthreads();
        drain();
        if (bin_c) {
            atomicAdd(&out.hsumq[(size_t)cur * kBuckets + tid], (unsigned long long)bin_q);
            atomicAdd(&out.hcnt[(size_t)cur * kBuckets + tid], bin_c);
        }
        bin_q = 0;
        bin_c = 0;
        if (__syncthreads_or((int)(far.lo_cnt | far.hi_cnt))) {      // also the barrier after the drain
            double c_lo = (double)far.lo_cnt, c_hi = (double)far.hi_cnt;
            block_sum2(far.lo_sum, far.hi_sum, s_red);
            block_sum2(c_lo, c_hi, s_red);
            if (tid == 0) {
                if (c_lo > 0.0) {
                    atomicAdd(&out.osum[2 * (size_t)cur], far.lo_sum);
                    atomicAdd(&out.ocnt[2 * (size_t)cur], (unsigned long long)c_lo);
                }
                if (c_hi > 0.0) {
                    atomicAdd(&out.osum[2 * (size_t)cur + 1], far.hi_sum);
                    atomicAdd(&out.ocnt[2 * (size_t)cur + 1], (unsigned long long)c_hi);
                }
            }
            far = FarSums();
        }
    };
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
            if (s != cur) {
                if (cur != kNoSegment) flush_segment();
                cur = s;
                src.enter_segment(s);
                bs = bin_scale(qp[s].lo, qp[s].inv_w);
            }
            auto single = [&](uint64_t lo, uint64_t hi) {
                for (uint64_t i = lo + tid; i < hi; i += kThreads)
                    codes[i] = kBins ? (uint8_t)code_and_bin(src.value1(i), bs, s_bin, kCopies, far)
                                     : (uint8_t)code_only(src.value1(i), bs);
                pending += (uint32_t)(hi - lo);
            };
            auto drain_if_due = [&]() {
                if (kBins && pending >= kDrainAfter) {
                    __syncthreads();
                    drain();
                    __syncthreads();
                }
            };
            uint64_t base = aligned_start(pos, sub_end, phase);
            single(pos, base);                   // fewer than 128 elements
            for (; base + kIter <= sub_end; base += kIter) {
                typename Src::Raw raw[kUnroll];
#pragma unroll
                for (int j = 0; j < kUnroll; ++j)
                    raw[j] = src.fetch4(base + (uint64_t)(j * kThreads + tid) * kVec);
#pragma unroll
                for (int j = 0; j < kUnroll; ++j) {
                    const f32x4 v = src.value4(raw[j]);
                    const uint32_t packed = kBins ? code_and_bin4(v, bs, s_bin, kCopies, far) : code_only4(v, bs);
                    if (phased)
                        s_stage[staged * (kIter / 4) + j * kThreads + tid] = packed;
                    else
                        st_u8x4(codes + base + (uint64_t)(j * kThreads + tid) * kVec, packed);
                }
                if (phased) {
                    if (tid == 0) s_stage_at[staged] = base;
                    ++staged;
                    bool write_now = staged == kStage;
                    if (!write_now)
                        write_now = __syncthreads_or(
                            tid == 0 ? (uint32_t)(wall_clock64() % phase_cfg.period) < phase_cfg.window : 0);
                    if (write_now) write_staged();
                }
                pending += kIter;
                drain_if_due();
            }
            single(base, sub_end);               // fewer than kIter elements
            drain_if_due();
            pos = sub_end;
        }
    }
    if (staged) write_staged();
    if (cur != kNoSegment) flush_segment();
}

}  // namespace diloco
