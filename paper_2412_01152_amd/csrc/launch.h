// Host-side launch plumbing shared by the translation units of the library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_common.h"

namespace diloco {

// Everything the two quantising passes share for one call.
struct Pass {
    uint64_t N;
    uint32_t T;
    const uint64_t* seg;        // device, [T+1]
    double* stats;              // device, [T][2]
    float* pivot;               // device, [T]
    unsigned long long* hsumq;  // device, [T][256]
    unsigned long long* hcnt;   // device, [T][256]
    double* osum;               // device, [T][2]
    unsigned long long* ocnt;   // device, [T][2]
    unsigned long long* counters;   // device, [kNumCounters], zero at the start of the call
    int num_cus;
    WritePhase write_phase;     // when pass B writes its staged codes
    hipStream_t stream;
};

struct ReduceArgs {
    const uint8_t* codes[DILOCO_MAX_PEERS];
    const float* luts[DILOCO_MAX_PEERS];
    uint32_t W;
    const float* local;
    float div;        // divisor (true_div) or its exact reciprocal
    bool true_div;
};

// Optional HIP events recorded around the streaming passes (benchmark instrumentation); all null
// unless the calling thread asked for them.
struct PassEvents {
    hipEvent_t ev[4];
};
PassEvents& pass_events();
inline hipError_t mark(int which, hipStream_t stream) {
    hipEvent_t e = pass_events().ev[which];
    return e ? hipEventRecord(e, stream) : hipSuccess;
}

// Resident blocks per compute unit of a kernel, looked up once per process (the initialisation of a
// function-local static is thread-safe).
template <auto Kernel>
inline int resident_blocks_per_cu() {
    static const int occ = [] {
        int v = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, Kernel, kThreads, 0) != hipSuccess || v < 1) v = 4;
        return v;
    }();
    return occ;
}

// Launch shape of a streaming pass: all blocks resident (grid = CUs x resident blocks, fewer when
// the buffer is small), chunks of at most max_chunk_iters block iterations claimed dynamically.
struct Grid {
    uint32_t blocks;
    Work work;
};
// Elements per claim, in block iterations of 4,096 elements (upper limits; small buffers get
// smaller chunks so that every block still sees about 16 of them).  A claim costs about 20 ns at
// the one counter, which bounds how short a chunk may be: a pass that moves 5 bytes per element takes
// 8.5 ms at 8 iterations and 10.5 ms at 4, one that moves 20 and more is still faster at 4.  Measured inside
// one process at the 10B size: passes that only read run fastest with long chunks (stage 1 pass A:
// 12.12 ms at 32, 11.73 ms at 128), passes that also write with short ones, which keep the blocks'
// working set within a narrower window of addresses (stage 1 pass B: 15.32 ms at 32, 14.94 ms at 8;
// bf16: 12.99 -> 12.42 ms; pass A of the reduce when it stores the accumulation, W = 14: 33.4 ms at
// 32, 32.0 ms at 4).  Pass B of the reduce source, which recomputes the values from W code streams, sits
// in between (W = 4, four resident blocks: 9.56 ms at 8, 9.36 at 16, 9.48 at 32, 9.60 at 64).
constexpr uint64_t kChunkItersRead = 128;
constexpr uint64_t kChunkItersWrite = 8;
// Pass A of the reduce when it stores the accumulation: the more bytes an element moves, the longer
// a chunk lasts and the shorter it may be before the counter binds (13 codes + fp32 addend in and
// fp32 out, 21 B/element, ring-chunk calls: 45.7 ms at 4 iterations, 43.9 at 2; 4 codes in and fp32
// out, 8 B/element: 22.9 ms at 4, 26.4 at 2).
inline uint64_t chunk_iters_store_acc(uint32_t W, bool has_local) {
    return W + (has_local ? 4u : 0u) + 4u >= 20u ? 2 : 4;
}
constexpr uint64_t kChunkItersOuter = 2;      // coded form, 2 blocks per CU: 26.84 ms at 8, 26.62 at 4, 26.04 at 2, 33.0 at 1
constexpr uint64_t kChunkItersReduceWrite = 16;
// Blocks per compute unit where fewer than fit run faster (fewer concurrent streams for the memory
// system): the pass that only reads two fp32 streams (11.62 ms with the 7 that fit, 11.36 with 2,
// 11.27 with 1) and the outer step (26.96 ms with the 6 that fit, 26.64 with 2, 27.18 with 1).  The
// Pass B of the streaming sources: 4 (what the staged codes leave room for anyway; the stored-array
// source, which does not stage, 8.54 ms with the 6 that fit, 8.35 with 4).  The reduce-source
// kernels are fastest with all the blocks their LDS use admits (3 or 4): their table look-ups need
// the waves.
// Pass A of the reduce when it also stores the fp32 accumulation: a write stream next to W byte
// streams wants few blocks while the table look-ups still find enough waves (10B buffer, 4 blocks
// resident: W = 4: 14.0 ms with all of them, 13.4 with 2; W = 8: 20.5 / 19.4; W = 10: 24.1 with 4,
// 23.7 with 3, 28.7 with 2; W = 14: 30.8 with the 3 that fit, 38.8 with 2).
inline int blocks_per_cu_store_acc(uint32_t W) { return W <= 8 ? 2 : 3; }
constexpr int kBlocksPerCuStreamRead = 1;
constexpr int kBlocksPerCuStreamWrite = 4;
constexpr int kBlocksPerCuOuter = 2;
inline uint32_t host_phase(const void* p, int elem_bytes) {
    return (uint32_t)((uintptr_t)p / (uintptr_t)elem_bytes) & (kAlignElems - 1);
}
inline void set_phase(Work& w, uint64_t N, uint32_t phase) {
    w.phase = phase;
    w.origin = (kAlignElems - phase) & (kAlignElems - 1);
    const uint64_t body = N > w.origin ? N - w.origin : 0;
    w.num_chunks = (body + w.chunk - 1) / w.chunk;
    if (w.num_chunks < 1) w.num_chunks = 1;
}
inline Grid plan_grid(uint64_t N, int num_cus, int blocks_per_cu, unsigned long long* counter, uint32_t phase,
                      uint64_t max_chunk_iters) {
    Grid g;
    const uint64_t resident = (uint64_t)num_cus * (uint64_t)blocks_per_cu;
    uint64_t iters = (N + kIter - 1) / kIter;
    if (iters < 1) iters = 1;
    // about 16 chunks per block when the buffer is small, but never so short that the counter
    // becomes the bottleneck (a quarter of a million claims take 5 ms, whatever the kernel does)
    const uint64_t min_chunk_iters = max_chunk_iters < 8 ? max_chunk_iters : 8;
    uint64_t chunk_iters = iters / (resident * 16);
    if (chunk_iters < min_chunk_iters) chunk_iters = min_chunk_iters;
    if (chunk_iters > max_chunk_iters) chunk_iters = max_chunk_iters;
    g.work.counter = counter;
    g.work.chunk = chunk_iters * kIter;
    set_phase(g.work, N, phase);
    g.blocks = (uint32_t)(g.work.num_chunks < resident ? g.work.num_chunks : resident);
    if (g.blocks < 1) g.blocks = 1;
    return g;
}

// Stage 2 launchers; the W values are spread over several translation units (groups of W) so they
// compile in parallel.  Each returns hipErrorInvalidValue for a W outside its group.
#define DILOCO_DECLARE_REDUCE_GROUP(G)                                                           \
    hipError_t launch_reduce_stats_g##G(const ReduceArgs& a, const Pass& p, float* acc_out);    \
    hipError_t launch_reduce_quant_g##G(const ReduceArgs& a, const Pass& p,                     \
                                        const diloco_qparams* qp, uint8_t* codes);
DILOCO_DECLARE_REDUCE_GROUP(0)
DILOCO_DECLARE_REDUCE_GROUP(1)
DILOCO_DECLARE_REDUCE_GROUP(2)
DILOCO_DECLARE_REDUCE_GROUP(3)
#undef DILOCO_DECLARE_REDUCE_GROUP

// One contiguous share per block, no counter: what the outer step falls back to when its fp32 form
// is called without a workspace (1-3 % slower than claimed chunks).
inline Grid plan_static(uint64_t N, int num_cus, int blocks_per_cu, uint32_t phase) {
    Grid g;
    uint64_t want = (uint64_t)num_cus * (uint64_t)blocks_per_cu;
    uint64_t iters = (N + kIter - 1) / kIter;
    if (iters < 1) iters = 1;
    if (want > iters) want = iters;
    g.work.counter = nullptr;
    g.work.chunk = (iters + want - 1) / want * kIter;
    set_phase(g.work, N, phase);
    g.blocks = (uint32_t)g.work.num_chunks;
    if (g.blocks < 1) g.blocks = 1;
    return g;
}

inline int reduce_group_of(uint32_t W) { return W <= 4 ? 0 : (W <= 8 ? 1 : (W <= 12 ? 2 : 3)); }

}  // namespace diloco
