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
    bool bins;                  // pass B also sums the buckets (false: the codebook needs no sums)
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
// smaller chunks so that every block still sees about 16 of them).  A claim costs a fixed time at
// the one counter, which bounds how short a chunk may be; above that bound, passes that only read
// run fastest with long chunks, passes that also write with short ones (the blocks' working set
// then stays within a narrow window of addresses), and the more bytes an element moves the shorter
// the best chunk.  All values below were chosen by measurement at the 10B size.
constexpr uint64_t kChunkItersRead = 128;
constexpr uint64_t kChunkItersWrite = 8;
// Pass A of the reduce when it stores the accumulation: 2 iterations when an element moves 20 bytes
// or more (13 codes + fp32 addend in, fp32 out), else 4.
inline uint64_t chunk_iters_store_acc(uint32_t W, bool has_local) {
    return W + (has_local ? 4u : 0u) + 4u >= 20u ? 2 : 4;
}
constexpr uint64_t kChunkItersOuter = 2;
constexpr uint64_t kChunkItersReduceWrite = 16;
constexpr uint64_t kChunkItersReduceNoBins = 8;      // pass B of the reduce when the codebook needs no bucket sums
// Blocks per compute unit where fewer than fit run faster (fewer concurrent streams for the memory
// system): one for the pass that only reads two fp32 streams, two for the outer step, four for
// pass B of the streaming sources.  The reduce-source kernels are fastest with all the blocks their
// LDS use admits (their table look-ups need the waves), except pass A when it also stores the fp32
// accumulation: a write stream next to W byte streams wants few blocks, 2 up to W = 8 and 3 beyond.
inline int blocks_per_cu_store_acc(uint32_t W) { return W <= 8 ? 2 : 3; }
constexpr int kBlocksPerCuStreamRead = 1;
constexpr int kBlocksPerCuStreamWrite = 4;
constexpr int kBlocksPerCuOuter = 2;
constexpr int kBlocksPerCuReduceNoBins = 3;
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
