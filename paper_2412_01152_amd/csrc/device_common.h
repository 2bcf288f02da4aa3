// Device-side building blocks shared by the gfx950 kernels of this library: alignment-tolerant
// vector access, the block's share of the flat buffer, segment lookup, wave64 / block reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/diloco_mi355.h"

namespace diloco {

constexpr int kThreads = 256;                       // 4 wave64 per block; also the number of buckets
constexpr int kVec = 4;                             // consecutive elements per lane per load
constexpr int kUnroll = 4;                          // loads in flight per stream per lane
// Copies of the 256 LDS bins in pass B (a lane uses copy lane % copies): one is enough where the
// pass waits for two fp32 streams; the reduce source issues its atomics in denser bursts and runs
// measurably faster with sixteen.
constexpr int kBinCopiesStream = 1;
constexpr int kBinCopiesReduce = 16;
// Iterations of codes (4 KiB each) a block of pass B can hold back in LDS, and the write window of
// the staged codes in microseconds: the first kWriteWindowUs of every kWritePeriodUs.
constexpr int kStageIters = 8;
constexpr int kWritePeriodUs = 40;
constexpr int kWriteWindowUs = 10;
constexpr uint64_t kMinPhasedElems = 1ull << 27;   // staging pays from a few hundred million elements on
struct WritePhase {
    uint32_t period;   // in ticks of wall_clock64(); 0 = write every iteration's codes at once
    uint32_t window;   // the first `window` ticks of each period are the write window
};
constexpr int kIter = kThreads * kVec * kUnroll;    // elements one block consumes per iteration
constexpr int kBuckets = 256;
constexpr uint32_t kNoSegment = 0xffffffffu;
// Fixed-point bucket sums: a 64-bit LDS bin holds {count : 16 bits, sum of addends : 48 bits}.
// An offset from the bucket centre is at most one bucket width; scaled by 2^21 / width and added to
// 1.5 * 2^23 in fp32 it becomes an integer in the low mantissa bits of the result, and the bit
// pattern of that float (0x4B400000 + round(offset * 2^21 / width), below 2^31) is the addend: no
// masking per element, the constant part is taken out again, count times, when a bin is drained.
constexpr int kOffsetBits = 21;
constexpr float kRoundMagic = 12582912.0f;          // 1.5 * 2^23: adding it rounds to an integer
constexpr long long kAddendBase = 0x4B400000ll;     // bit pattern of kRoundMagic
constexpr int kCountShift = 48;
constexpr int kFlushIters = 12;                     // the bins are drained once 12 iterations are in
// the count of binned elements is checked after every iteration and every ragged tail (< kIter
// elements) and a head (< 128) may follow unchecked, so fewer than (kFlushIters + 2) * kIter
// elements sit in the bins at any time: their count must fit 16 bits, their sum 48
static_assert((long long)(kFlushIters + 2) * kIter < (1ll << (64 - kCountShift)), "bin count overflow");
static_assert((long long)(kFlushIters + 2) * kIter * (1ll << 31) <= (1ll << kCountShift), "bin sum overflow");

// Vector types that promise only element alignment: gfx950 global memory instructions accept
// any byte address, so one dwordx4 / dwordx2 / dword access is emitted whatever the pointer's
// alignment (chunk boundaries of a ring all-reduce are arbitrary element offsets).
typedef float f32x4_u __attribute__((ext_vector_type(4), aligned(4)));
typedef uint16_t u16x4_u __attribute__((ext_vector_type(4), aligned(2)));
typedef uint32_t u32_u __attribute__((aligned(1)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_u __attribute__((ext_vector_type(4), aligned(1)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Every array here is streamed once per pass, so loads and stores carry the non-temporal hint
// (measured on MI355X: about 12 % more read bandwidth than plain loads on a pure read stream).
#define DILOCO_NT 1
__device__ __forceinline__ f32x4 ld_f32x4(const float* p) {
#if DILOCO_NT
    return __builtin_nontemporal_load((const f32x4_u*)p);
#else
    return *(const f32x4_u*)p;
#endif
}
__device__ __forceinline__ void st_f32x4(float* p, f32x4 v) {
#if DILOCO_NT
    __builtin_nontemporal_store(v, (f32x4_u*)p);
#else
    *(f32x4_u*)p = v;
#endif
}
__device__ __forceinline__ uint32_t ld_u8x4(const uint8_t* p) {
#if DILOCO_NT
    return __builtin_nontemporal_load((const u32_u*)p);
#else
    return *(const u32_u*)p;
#endif
}
__device__ __forceinline__ void st_u8x4(uint8_t* p, uint32_t v) {
#if DILOCO_NT
    __builtin_nontemporal_store(v, (u32_u*)p);
#else
    *(u32_u*)p = v;
#endif
}

__device__ __forceinline__ void st_u8x16(uint8_t* p, u32x4 v) {
#if DILOCO_NT
    __builtin_nontemporal_store((u32x4_u)v, (u32x4_u*)p);
#else
    *(u32x4_u*)p = (u32x4_u)v;
#endif
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ f32x4 ld_bf16x4(const uint16_t* p) {
#if DILOCO_NT
    u16x4_u h = __builtin_nontemporal_load((const u16x4_u*)p);
#else
    u16x4_u h = *(const u16x4_u*)p;
#endif
    f32x4 r;
    r[0] = bf16_bits_to_f32(h[0]);
    r[1] = bf16_bits_to_f32(h[1]);
    r[2] = bf16_bits_to_f32(h[2]);
    r[3] = bf16_bits_to_f32(h[3]);
    return r;
}

// fp32 -> bf16 bit pattern, round to nearest even, NaN kept quiet.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((b >> 16) | 0x40u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

// Work distribution of the streaming passes.  The flat buffer [0, N) is cut into chunks of
// `chunk` elements (a multiple of kIter); the resident blocks claim chunks in address order from a
// global counter until none is left.  Blocks of one launch progress at very different speeds on
// this chip (measured: up to 2.7x apart in a static partition, so the slowest blocks ran alone
// for a third of the kernel), which a static split turns into idle compute units; claiming keeps
// every block busy to the end.  The next claim is issued before the current chunk is processed,
// so its latency is hidden.  Every wave leaves the loop when the counter passes num_chunks.
struct Work {
    unsigned long long* counter;   // device, zero before the launch; nullptr: chunks are dealt
                                   // round-robin (block b takes b, b + grid, ...) without a counter
    uint64_t chunk;                // elements per claim
    uint64_t num_chunks;
    uint32_t phase;                // reference stream's address in elements, modulo kAlignElems
    uint32_t origin;               // (kAlignElems - phase) % kAlignElems: chunk c >= 1 starts at
                                   // origin + c * chunk, a line-aligned position; chunk 0 at element 0
};
struct Share {
    uint64_t begin, end;
};
// The element range of claim c (c < w.num_chunks): chunk 0 starts at element 0 and also takes the
// elements in front of the origin, chunk c >= 1 starts at origin + c * chunk.
__host__ __device__ __forceinline__ Share claim_range(const Work& w, unsigned long long c, uint64_t N) {
    Share sh;
    sh.begin = c ? w.origin + c * w.chunk : 0;
    const uint64_t e = w.origin + (c + 1) * w.chunk;
    sh.end = e < N ? e : N;
    return sh;
}
struct Claimer {
    unsigned long long next;
    __device__ __forceinline__ explicit Claimer(const Work& w) : next(blockIdx.x) {
        if (w.counter && threadIdx.x == 0) next = atomicAdd(w.counter, 1ull);
    }
    // Block-uniform.  `slot` is one 64-bit word of LDS.
    __device__ __forceinline__ bool claim(const Work& w, uint64_t N, Share& sh, unsigned long long* slot) {
        if (threadIdx.x == 0) *slot = next;
        __syncthreads();
        const unsigned long long c = *slot;
        __syncthreads();
        if (c >= w.num_chunks) return false;
        if (!w.counter)
            next += gridDim.x;
        else if (threadIdx.x == 0)
            next = atomicAdd(w.counter, 1ull);
        sh = claim_range(w, c, N);
        return true;
    }
};

// Pointers need only element alignment, but the streaming loops run about a fifth faster when a
// wave's accesses start on 128-byte lines (measured: views shifted by 1, 3, 5 or 16 elements all
// cost the same 15-20 %, so it is the cache-line straddling and the partial-line writes that hurt,
// not the width of the vector access).  Each piece of work therefore starts with up to 127 single
// elements, until element index + phase is a multiple of 128, where phase is the reference
// stream's address in elements modulo 128 (taken by the host from the pointer it passes; chunk
// starts are shifted to the same phase).  Streams that share the reference's phase (views of
// line-aligned buffers at the same element offset) become line-aligned, byte codes included;
// any other stream is still accessed correctly, just unaligned.
constexpr uint32_t kAlignElems = 128;
__device__ __forceinline__ uint64_t aligned_start(uint64_t pos, uint64_t end, uint32_t phase) {
    const uint32_t mis = (uint32_t)(pos + phase) & (kAlignElems - 1);
    const uint64_t a = mis ? pos + (kAlignElems - mis) : pos;
    return a < end ? a : end;
}

// Index of the segment that holds element `pos` (pos < seg[T]): the smallest s with seg[s+1] > pos.
__device__ __forceinline__ uint32_t find_segment(const uint64_t* __restrict__ seg, uint32_t T,
                                                 uint64_t pos) {
    uint32_t lo = 0, hi = T - 1;
    while (lo < hi) {
        uint32_t mid = (lo + hi) >> 1;
        if (seg[mid + 1] > pos)
            hi = mid;
        else
            lo = mid + 1;
    }
    return lo;
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Sum of two per-thread doubles over the block; result valid in thread 0.  `red` is 8 doubles of LDS.
__device__ __forceinline__ void block_sum2(double& a, double& b, double* red) {
    a = wave_sum(a);
    b = wave_sum(b);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) {
        red[wave] = a;
        red[4 + wave] = b;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        a = (red[0] + red[1]) + (red[2] + red[3]);
        b = (red[4] + red[5]) + (red[6] + red[7]);
    }
}

// fp32 bucket width and bucket centre used for the codebook sums: the kernel accumulates
// (x - centre_k), whose magnitude is half a bucket, instead of x; the finalising kernel adds
// centre_k back in fp64.  Both must use exactly these two functions.
__device__ __forceinline__ float bucket_width(float inv_w) {
    return inv_w > 0.0f ? __fdiv_rn(1.0f, inv_w) : 0.0f;
}
__device__ __forceinline__ float bucket_centre0(float lo, float w) { return __fmaf_rn(0.5f, w, lo); }
__device__ __forceinline__ float bucket_centre(float kf, float centre0, float w) {
    return __fmaf_rn(kf, w, centre0);
}
// Bucket index of Section 2.2's quantiser, as a float (0.0 .. 255.0): floor((x - lo) / width)
// clipped to [0, 255], with the subtraction and the multiplication by the reciprocal width as two
// separately rounded fp32 operations (never contracted into a fused multiply-add).  Anything <= 0
// or NaN clamps to bucket 0, anything >= 255 to bucket 255.
__device__ __forceinline__ float bucket_of_f(float x, float lo, float inv_w) {
    const float t = __fmul_rn(__fsub_rn(x, lo), inv_w);
    return __builtin_amdgcn_fmed3f(__builtin_floorf(t), 0.0f, 255.0f);
}
// Factor that turns an offset from the bucket centre into fixed point: 2^21 / width (0 when the
// segment is degenerate or the factor would overflow; then every non-zero offset goes the fp64 way).
__device__ __forceinline__ float offset_scale(float inv_w) {
    const float s = __fmul_rn(inv_w, (float)(1 << kOffsetBits));
    return (inv_w > 0.0f && s <= 3.0e38f) ? s : 0.0f;
}

// Device scratch layout (all offsets in bytes from a 256-byte aligned base).
struct WorkspaceLayout {
    size_t seg, stats, pivot, hsumq, hcnt, osum, ocnt, counters, total;
};
constexpr int kNumCounters = 4;     // chunk counters: pass A, pass B, outer step, spare
__host__ __device__ constexpr size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
__host__ constexpr WorkspaceLayout workspace_layout(uint32_t T) {
    WorkspaceLayout L{};
    size_t o = 0;
    L.seg = o;
    o = align_up(o + sizeof(uint64_t) * ((size_t)T + 1), 256);
    L.stats = o;
    o = align_up(o + sizeof(double) * 2 * (size_t)T, 256);
    L.pivot = o;
    o = align_up(o + sizeof(float) * (size_t)T, 256);
    L.hsumq = o;
    o = align_up(o + sizeof(unsigned long long) * kBuckets * (size_t)T, 256);
    L.hcnt = o;
    o = align_up(o + sizeof(unsigned long long) * kBuckets * (size_t)T, 256);
    L.osum = o;
    o = align_up(o + sizeof(double) * 2 * (size_t)T, 256);
    L.ocnt = o;
    o = align_up(o + sizeof(unsigned long long) * 2 * (size_t)T, 256);
    L.counters = o;
    o = align_up(o + sizeof(unsigned long long) * kNumCounters, 256);
    L.total = o;
    return L;
}

}  // namespace diloco
