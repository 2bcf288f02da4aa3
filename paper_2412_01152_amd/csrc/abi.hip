// Host side of the C ABI declared in include/diloco_mi355.h: argument checks, scratch layout,
// and the launch sequence of each call.  Everything is enqueued on the caller's stream; nothing
// here allocates, frees or waits for the device.
#include <math.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <string.h>

#include "finalize_kernels.h"
#include "kernels.h"
#include "launch.h"
#include "outer_kernel.h"

using namespace diloco;

namespace diloco {
PassEvents& pass_events() {
    static thread_local PassEvents e = {{nullptr, nullptr, nullptr, nullptr}};
    return e;
}
}  // namespace diloco

namespace {

// Segment offsets travel to the device inside kernel arguments (no staging copy, no host
// synchronisation, nothing but kernels on the stream).  A launch's arguments may take 4 KiB: up to
// 480 offsets go up as they are, in one launch.  Longer tables go up as 32-bit segment lengths,
// 960 per launch, and one more kernel turns them into offsets with a prefix sum (66 + 1 launches at
// the largest table the library takes); a table with a segment of 2^32 elements or more falls back
// to 64-bit offsets, 480 per launch.
constexpr uint32_t kOffsetsPerLaunch = 480;
constexpr uint32_t kLengthsPerLaunch = 960;
struct OffsetBlock {
    uint64_t v[kOffsetsPerLaunch];
};
struct LengthBlock {
    uint32_t v[kLengthsPerLaunch];
};
template <class Block>
__global__ void upload_block_kernel(Block blk, uint64_t* dst, uint32_t count) {
    for (uint32_t i = threadIdx.x; i < count; i += blockDim.x) dst[i] = blk.v[i];
}

// In-place inclusive prefix sum of v[0 .. count) by one block of 1,024 threads: every thread sums
// a contiguous slice, the 1,024 slice sums are scanned with wave shuffles, every thread rewrites
// its slice.
__global__ __launch_bounds__(1024) void scan_offsets_kernel(uint64_t* v, uint32_t count) {
    __shared__ uint64_t s_wave[16];
    const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t per = (count + 1023) / 1024;
    const uint32_t a = tid * per < count ? tid * per : count;
    const uint32_t b = a + per < count ? a + per : count;
    uint64_t sum = 0;
    for (uint32_t i = a; i < b; ++i) sum += v[i];
    uint64_t incl = sum;                                  // inclusive scan of the slice sums within the wave
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint64_t up = __shfl_up(incl, o, 64);
        if (lane >= (uint32_t)o) incl += up;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    uint64_t before = incl - sum;                         // everything in front of this thread's slice
    for (uint32_t w = 0; w < wave; ++w) before += s_wave[w];
    for (uint32_t i = a; i < b; ++i) {
        before += v[i];
        v[i] = before;
    }
}

hipError_t upload_offsets(const uint64_t* host, uint32_t count, uint64_t* dst, hipStream_t stream) {
    bool narrow = count > kOffsetsPerLaunch;
    for (uint32_t i = 1; narrow && i < count; ++i) narrow = host[i] - host[i - 1] <= 0xffffffffull;
    if (!narrow) {
        for (uint32_t first = 0; first < count; first += kOffsetsPerLaunch) {
            OffsetBlock blk;
            const uint32_t c = count - first < kOffsetsPerLaunch ? count - first : kOffsetsPerLaunch;
            memcpy(blk.v, host + first, sizeof(uint64_t) * c);
            hipLaunchKernelGGL(upload_block_kernel<OffsetBlock>, dim3(1), dim3(256), 0, stream, blk, dst + first, c);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    // dst[0] = host[0] (= 0), dst[i] = length of segment i - 1; then the prefix sum
    for (uint32_t first = 0; first < count; first += kLengthsPerLaunch) {
        LengthBlock blk;
        const uint32_t c = count - first < kLengthsPerLaunch ? count - first : kLengthsPerLaunch;
        for (uint32_t i = 0; i < c; ++i) {
            const uint32_t g = first + i;
            blk.v[i] = g == 0 ? (uint32_t)host[0] : (uint32_t)(host[g] - host[g - 1]);
        }
        hipLaunchKernelGGL(upload_block_kernel<LengthBlock>, dim3(1), dim3(256), 0, stream, blk, dst + first, c);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(scan_offsets_kernel, dim3(1), dim3(1024), 0, stream, dst, count);
    return hipGetLastError();
}

bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }

int32_t check_segments(const uint64_t* seg, uint32_t T, uint64_t N) {
    if (T == 0 || T > DILOCO_MAX_SEGMENTS) return DILOCO_ERR_SIZE;
    if (!seg) return DILOCO_ERR_NULL;
    if (seg[0] != 0 || seg[T] != N) return DILOCO_ERR_SIZE;
    for (uint32_t s = 0; s < T; ++s)
        if (seg[s + 1] < seg[s]) return DILOCO_ERR_SIZE;
    return DILOCO_OK;
}

// Timing of pass B's staged code writes.  The product picks it by size alone (staged from
// kMinPhasedElems elements on, with the built-in period and window); diloco_tune_write_phase lets a
// test or a benchmark force another choice.  One packed word, so a reader never sees half an update:
// bit 63 = override active, bits 32..62 = period in us (0 = write at once), bits 0..31 = window in us.
std::atomic<uint64_t> g_write_phase_override{0};
constexpr uint64_t kOverrideActive = 1ull << 63;

// Write window of pass B in ticks of the device's constant-rate clock; period 0 (write at once)
// when the clock rate cannot be read.
WritePhase write_phase_ticks(int period_us, int window_us) {
    WritePhase w = {0, 0};
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return w;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz < 1000) return w;
    w.period = (uint32_t)((long long)khz * period_us / 1000);
    w.window = (uint32_t)((long long)khz * window_us / 1000);
    return w;
}

WritePhase choose_write_phase(uint64_t N) {
    const uint64_t o = g_write_phase_override.load(std::memory_order_relaxed);
    if (o & kOverrideActive) {
        const int period_us = (int)((o >> 32) & 0x7fffffffu), window_us = (int)(o & 0xffffffffu);
        return period_us ? write_phase_ticks(period_us, window_us) : WritePhase{0, 0};
    }
    // a launch shorter than a few periods only loses by waiting for its window
    return N >= kMinPhasedElems ? write_phase_ticks(kWritePeriodUs, kWriteWindowUs) : WritePhase{0, 0};
}

int32_t num_compute_units(int* out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int32_t)e;
    e = hipDeviceGetAttribute(out, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return (int32_t)e;
    if (*out < 1) *out = 1;
    return 0;
}

// Uploads the offsets, clears the accumulators, and fills in the Pass record.
int32_t begin_pass(Pass& p, uint64_t N, uint32_t T, const uint64_t* seg_host, void* workspace,
                   size_t workspace_bytes, hipStream_t stream, bool bins) {
    if (!workspace) return DILOCO_ERR_NULL;
    if (misaligned(workspace, 256)) return DILOCO_ERR_ALIGN;
    const WorkspaceLayout L = workspace_layout(T);
    if (workspace_bytes < L.total) return DILOCO_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    p.N = N;
    p.T = T;
    p.seg = (const uint64_t*)(ws + L.seg);
    p.stats = (double*)(ws + L.stats);
    p.pivot = (float*)(ws + L.pivot);
    p.hsumq = (unsigned long long*)(ws + L.hsumq);
    p.hcnt = (unsigned long long*)(ws + L.hcnt);
    p.osum = (double*)(ws + L.osum);
    p.ocnt = (unsigned long long*)(ws + L.ocnt);
    p.counters = (unsigned long long*)(ws + L.counters);
    p.stream = stream;
    p.bins = bins;
    int32_t rc = num_compute_units(&p.num_cus);
    if (rc) return rc;
    p.write_phase = choose_write_phase(N);
    hipError_t e = upload_offsets(seg_host, T + 1, (uint64_t*)(ws + L.seg), stream);
    if (e != hipSuccess) return (int32_t)e;
    const size_t words = (L.total - L.stats) / sizeof(uint64_t);
    const unsigned blocks = (unsigned)((words + 255) / 256 < 1024 ? (words + 255) / 256 : 1024);
    hipLaunchKernelGGL(zero_kernel, dim3(blocks), dim3(256), 0, stream, (uint64_t*)(ws + L.stats), words);
    e = hipGetLastError();
    return e == hipSuccess ? 0 : (int32_t)e;
}

// The quantiser's two knobs; the paper's are {6, bucket averages}.
struct QuantVariant {
    double range_sigmas;
    uint32_t codebook;
};
constexpr QuantVariant kPaperQuantiser = {6.0, DILOCO_CODEBOOK_MEAN};

int32_t check_variant(double range_sigmas, uint32_t codebook) {
    if (!(range_sigmas >= DILOCO_MIN_RANGE_SIGMAS && range_sigmas <= DILOCO_MAX_RANGE_SIGMAS)) return DILOCO_ERR_SIZE;
    if (codebook != DILOCO_CODEBOOK_MEAN && codebook != DILOCO_CODEBOOK_MIDPOINT) return DILOCO_ERR_DTYPE;
    return DILOCO_OK;
}

hipError_t finalize_qparams(const Pass& p, const QuantVariant& v, diloco_qparams* qp) {
    hipLaunchKernelGGL(finalize_qparams_kernel, dim3((p.T + 255) / 256), dim3(256), 0, p.stream, p.seg, p.T,
                       p.stats, p.pivot, v.range_sigmas, qp);
    return hipGetLastError();
}

hipError_t finalize_lut(const Pass& p, const QuantVariant& v, const diloco_qparams* qp, float* lut) {
    hipLaunchKernelGGL(finalize_lut_kernel, dim3(p.T), dim3(kThreads), 0, p.stream, p.T, v.range_sigmas,
                       v.codebook, qp, p.hsumq, p.hcnt, p.osum, p.ocnt, lut);
    return hipGetLastError();
}

template <class Src>
hipError_t run_stats(const Src& src, const Pass& p, uint32_t phase) {
    hipLaunchKernelGGL(pivot_kernel<Src>, dim3((p.T + kPivotSegmentsPerBlock - 1) / kPivotSegmentsPerBlock),
                       dim3(kThreads), 0, p.stream, src, p.seg, p.T,
                       p.pivot);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr auto kernel = stats_kernel<Src, false>;
    Grid g = plan_grid(p.N, p.num_cus, kBlocksPerCuStreamRead, p.counters + 0, phase, kChunkItersRead);
    (void)mark(0, p.stream);
    hipLaunchKernelGGL(kernel, dim3(g.blocks), dim3(kThreads), 0, p.stream, src, p.seg, p.T, p.N,
                       g.work, p.stats, p.pivot, (float*)nullptr);
    e = hipGetLastError();
    (void)mark(1, p.stream);
    return e;
}

template <class Src, int kCopies>
hipError_t run_quant_as(const Src& src, const Pass& p, const diloco_qparams* qp, uint8_t* codes) {
    constexpr auto kernel = quant_kernel<Src, kCopies, Src::kStage>;
    Grid g = plan_grid(p.N, p.num_cus, std::min(resident_blocks_per_cu<kernel>(), kBlocksPerCuStreamWrite),
                       p.counters + 1, host_phase(codes, 1), kChunkItersWrite);
    (void)mark(2, p.stream);
    hipLaunchKernelGGL(kernel, dim3(g.blocks), dim3(kThreads), 0, p.stream, src, p.seg, p.T, p.N,
                       g.work, qp, codes, PassBOut{p.hsumq, p.hcnt, p.osum, p.ocnt}, p.write_phase);
    hipError_t e = hipGetLastError();
    (void)mark(3, p.stream);
    return e;
}
template <class Src>
hipError_t run_quant(const Src& src, const Pass& p, const diloco_qparams* qp, uint8_t* codes) {
    return p.bins ? run_quant_as<Src, kBinCopiesStream>(src, p, qp, codes) : run_quant_as<Src, 0>(src, p, qp, codes);
}

hipError_t reduce_stats(const ReduceArgs& a, const Pass& p, float* acc_out) {
    switch (reduce_group_of(a.W)) {
        case 0: return launch_reduce_stats_g0(a, p, acc_out);
        case 1: return launch_reduce_stats_g1(a, p, acc_out);
        case 2: return launch_reduce_stats_g2(a, p, acc_out);
        default: return launch_reduce_stats_g3(a, p, acc_out);
    }
}

hipError_t reduce_quant(const ReduceArgs& a, const Pass& p, const diloco_qparams* qp, uint8_t* codes) {
    switch (reduce_group_of(a.W)) {
        case 0: return launch_reduce_quant_g0(a, p, qp, codes);
        case 1: return launch_reduce_quant_g1(a, p, qp, codes);
        case 2: return launch_reduce_quant_g2(a, p, qp, codes);
        default: return launch_reduce_quant_g3(a, p, qp, codes);
    }
}

// Scratch of the entry point that takes no workspace argument: one file-scope device array per GPU,
// laid out like a caller's workspace for DILOCO_STATIC_MAX_SEGMENTS segments.  In host code the
// array's name is only a handle; its device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = workspace_layout(DILOCO_STATIC_MAX_SEGMENTS).total;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];            // device address of `scratch` on device d, or nullptr

// Device address of this device's copy of `scratch` (looked up at the first call on the device).
int32_t static_scratch(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int32_t)e;
    if (dev < 0 || dev >= kMaxDevices) return (int32_t)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int32_t)e;
        if (!p) return (int32_t)hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return DILOCO_OK;
}

#define DILOCO_TRY(expr)                             \
    do {                                             \
        hipError_t e_ = (expr);                      \
        if (e_ != hipSuccess) return (int32_t)e_;    \
    } while (0)

// counter == nullptr: one contiguous share per block; otherwise chunks claimed from the counter
// (zeroed here, on the stream).
template <int kOut>
hipError_t run_outer(float* theta, float* mom, const float* delta, const uint8_t* codes, const float* lut,
                     const uint64_t* seg, uint32_t T, uint64_t N, float lr, float beta, void* local_out,
                     int num_cus, unsigned long long* counter, hipStream_t stream) {
    if (counter) {
        hipLaunchKernelGGL(zero_kernel, dim3(1), dim3(64), 0, stream, (uint64_t*)counter, (size_t)1);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    const uint32_t phase = host_phase(theta, 4);
    hipError_t e;
    if (delta) {
        constexpr auto kernel = outer_fp32_kernel<kOut>;
        const int bpc = std::min(resident_blocks_per_cu<kernel>(), kBlocksPerCuOuter);
        Grid g = counter ? plan_grid(N, num_cus, bpc, counter, phase, kChunkItersOuter)
                         : plan_static(N, num_cus, bpc, phase);
        (void)mark(0, stream);
        hipLaunchKernelGGL(kernel, dim3(g.blocks), dim3(kThreads), 0, stream, theta, mom, delta, N,
                           g.work, lr, beta, local_out);
        e = hipGetLastError();
    } else {
        constexpr auto kernel = outer_coded_kernel<kOut>;
        const int bpc = std::min(resident_blocks_per_cu<kernel>(), kBlocksPerCuOuter);
        Grid g = counter ? plan_grid(N, num_cus, bpc, counter, phase, kChunkItersOuter)
                         : plan_static(N, num_cus, bpc, phase);
        (void)mark(0, stream);
        hipLaunchKernelGGL(kernel, dim3(g.blocks), dim3(kThreads), 0, stream, theta, mom, codes, lut, seg, T,
                           N, g.work, lr, beta, local_out);
        e = hipGetLastError();
    }
    (void)mark(1, stream);
    return e;
}

int32_t pseudograd_quantize_impl(const float* theta_outer, const void* theta_local, int32_t local_dtype,
                                 uint64_t N, const uint64_t* seg_offsets, uint32_t T, uint8_t* codes_out,
                                 float* lut_out, diloco_qparams* qparams_out, void* workspace,
                                 size_t workspace_bytes, hipStream_t stream, const QuantVariant& v) {
    if (local_dtype != DILOCO_DTYPE_FP32 && local_dtype != DILOCO_DTYPE_BF16) return DILOCO_ERR_DTYPE;
    if (!lut_out || !qparams_out) return DILOCO_ERR_NULL;
    if (N > 0 && (!theta_outer || !theta_local || !codes_out)) return DILOCO_ERR_NULL;
    int32_t rc = check_segments(seg_offsets, T, N);
    if (rc) return rc;
    if (misaligned(theta_outer, 4) || misaligned(theta_local, local_dtype == DILOCO_DTYPE_BF16 ? 2 : 4) ||
        misaligned(lut_out, 4) || misaligned(qparams_out, 8))
        return DILOCO_ERR_ALIGN;
    Pass p;
    rc = begin_pass(p, N, T, seg_offsets, workspace, workspace_bytes, stream, v.codebook == DILOCO_CODEBOOK_MEAN);
    if (rc) return rc;
    if (local_dtype == DILOCO_DTYPE_BF16) {
        SrcPseudoGrad<true> src{theta_outer, theta_local};
        if (N) DILOCO_TRY(run_stats(src, p, host_phase(theta_outer, 4)));
        DILOCO_TRY(finalize_qparams(p, v, qparams_out));
        if (N) DILOCO_TRY(run_quant(src, p, qparams_out, codes_out));
    } else {
        SrcPseudoGrad<false> src{theta_outer, theta_local};
        if (N) DILOCO_TRY(run_stats(src, p, host_phase(theta_outer, 4)));
        DILOCO_TRY(finalize_qparams(p, v, qparams_out));
        if (N) DILOCO_TRY(run_quant(src, p, qparams_out, codes_out));
    }
    DILOCO_TRY(finalize_lut(p, v, qparams_out, lut_out));
    return DILOCO_OK;
}

int32_t reduce_chunk_impl(const uint8_t* const* peer_codes, const float* const* peer_luts, uint32_t W,
                          const float* local_fp32, uint32_t divisor, uint64_t n, const uint64_t* seg_offsets,
                          uint32_t T, float* acc_out, uint8_t* codes_out, float* lut_out,
                          diloco_qparams* qparams_out, void* workspace, size_t workspace_bytes,
                          hipStream_t stream, const QuantVariant& v) {
    if (W > DILOCO_MAX_PEERS || (W == 0 && !local_fp32) || divisor == 0) return DILOCO_ERR_SIZE;
    if (W > 0 && (!peer_codes || !peer_luts)) return DILOCO_ERR_NULL;
    if (!lut_out || !qparams_out) return DILOCO_ERR_NULL;
    if (n > 0 && !codes_out) return DILOCO_ERR_NULL;
    int32_t rc = check_segments(seg_offsets, T, n);
    if (rc) return rc;
    ReduceArgs a;
    memset(&a, 0, sizeof a);
    a.W = W;
    for (uint32_t p = 0; p < W; ++p) {
        if (!peer_luts[p] || (n > 0 && !peer_codes[p])) return DILOCO_ERR_NULL;
        if (misaligned(peer_luts[p], 4)) return DILOCO_ERR_ALIGN;
        a.codes[p] = peer_codes[p];
        a.luts[p] = peer_luts[p];
    }
    if (misaligned(local_fp32, 4) || misaligned(acc_out, 4) || misaligned(lut_out, 4) ||
        misaligned(qparams_out, 8))
        return DILOCO_ERR_ALIGN;
    a.local = local_fp32;
    if ((divisor & (divisor - 1)) == 0) {
        a.true_div = false;          // multiplying by 2^-j rounds exactly like dividing by 2^j
        a.div = 1.0f / (float)divisor;
    } else {
        a.true_div = true;
        a.div = (float)divisor;
    }
    Pass p;
    rc = begin_pass(p, n, T, seg_offsets, workspace, workspace_bytes, stream, v.codebook == DILOCO_CODEBOOK_MEAN);
    if (rc) return rc;
    if (n) DILOCO_TRY(reduce_stats(a, p, acc_out));
    DILOCO_TRY(finalize_qparams(p, v, qparams_out));
    if (n) {
        if (acc_out) {
            SrcF32 src{acc_out};
            DILOCO_TRY(run_quant(src, p, qparams_out, codes_out));
        } else {
            DILOCO_TRY(reduce_quant(a, p, qparams_out, codes_out));
        }
    }
    DILOCO_TRY(finalize_lut(p, v, qparams_out, lut_out));
    return DILOCO_OK;
}

}  // namespace

extern "C" {

size_t diloco_workspace_bytes(uint32_t T) {
    if (T == 0 || T > DILOCO_MAX_SEGMENTS) return 0;
    return workspace_layout(T).total;
}

int32_t diloco_profile_passes(void* const* events) {
    PassEvents& pe = pass_events();
    for (int i = 0; i < 4; ++i) pe.ev[i] = events ? (hipEvent_t)events[i] : nullptr;
    return DILOCO_OK;
}

int32_t diloco_placement(uint64_t arena_bytes, uint64_t* offsets_out) {
    if (!offsets_out) return DILOCO_ERR_NULL;
    constexpr uint64_t kGiB = 1ull << 30, kAlign = 4096;
    if (arena_bytes < 3 * kAlign) return DILOCO_ERR_SIZE;
    const uint64_t third = arena_bytes / 3 / kAlign * kAlign;
    // the spacing at which the measured dependence on distance has levelled off, if the arena is large
    // enough for three groups that far apart; else a third of the arena
    const uint64_t gap = arena_bytes >= 216 * kGiB ? 100 * kGiB : third;
    const uint64_t lead = std::min<uint64_t>(4 * kGiB, third / 8) / kAlign * kAlign;
    offsets_out[0] = lead;
    offsets_out[1] = lead + gap;
    offsets_out[2] = lead + 2 * gap;
    return DILOCO_OK;
}

int32_t diloco_tune_write_phase(int32_t period_us, int32_t window_us) {
    if (period_us < 0) {                                  // back to the built-in choice by size
        g_write_phase_override.store(0, std::memory_order_relaxed);
        return DILOCO_OK;
    }
    if (period_us == 0) {                                 // write at once, at every size
        g_write_phase_override.store(kOverrideActive, std::memory_order_relaxed);
        return DILOCO_OK;
    }
    if (window_us < 1 || window_us > period_us || period_us > 1000000) return DILOCO_ERR_SIZE;
    g_write_phase_override.store(kOverrideActive | ((uint64_t)period_us << 32) | (uint64_t)window_us,
                                 std::memory_order_relaxed);
    return DILOCO_OK;
}

const char* diloco_strerror(int32_t code) {
    switch (code) {
        case DILOCO_OK: return "ok";
        case DILOCO_ERR_NULL: return "a required pointer is NULL";
        case DILOCO_ERR_SIZE: return "bad size, segment table, W or divisor";
        case DILOCO_ERR_ALIGN: return "a pointer is not aligned to its element type";
        case DILOCO_ERR_WORKSPACE: return "workspace too small (see diloco_workspace_bytes)";
        case DILOCO_ERR_DTYPE: return "unknown dtype flag";
        case DILOCO_ERR_STATIC_LIMIT:
            return "more segments than the library's static scratch holds (DILOCO_STATIC_MAX_SEGMENTS)";
        default: break;
    }
    if (code > 0) return hipGetErrorString((hipError_t)code);
    return "unknown error";
}

int32_t diloco_pseudograd_quantize(const float* theta_outer, const void* theta_local, int32_t local_dtype,
                                   uint64_t N, const uint64_t* seg_offsets, uint32_t T, uint8_t* codes_out,
                                   float* lut_out, diloco_qparams* qparams_out, void* workspace,
                                   size_t workspace_bytes, void* stream) {
    return pseudograd_quantize_impl(theta_outer, theta_local, local_dtype, N, seg_offsets, T, codes_out, lut_out,
                                    qparams_out, workspace, workspace_bytes, (hipStream_t)stream,
                                    kPaperQuantiser);
}

int32_t diloco_pseudograd_quantize_variant(const float* theta_outer, const void* theta_local,
                                           int32_t local_dtype, uint64_t N, const uint64_t* seg_offsets,
                                           uint32_t T, uint8_t* codes_out, float* lut_out,
                                           diloco_qparams* qparams_out, void* workspace, size_t workspace_bytes,
                                           void* stream, double range_sigmas, uint32_t codebook) {
    int32_t rc = check_variant(range_sigmas, codebook);
    if (rc) return rc;
    return pseudograd_quantize_impl(theta_outer, theta_local, local_dtype, N, seg_offsets, T, codes_out, lut_out,
                                    qparams_out, workspace, workspace_bytes, (hipStream_t)stream,
                                    QuantVariant{range_sigmas, codebook});
}

int32_t int8_reduce_chunk(const uint8_t* const* peer_codes, const float* const* peer_luts, uint32_t W,
                          const float* local_fp32, uint32_t divisor, uint64_t n, const uint64_t* seg_offsets,
                          uint32_t T, float* acc_out, uint8_t* codes_out, float* lut_out,
                          diloco_qparams* qparams_out, void* workspace, size_t workspace_bytes, void* stream) {
    return reduce_chunk_impl(peer_codes, peer_luts, W, local_fp32, divisor, n, seg_offsets, T, acc_out, codes_out,
                             lut_out, qparams_out, workspace, workspace_bytes, (hipStream_t)stream,
                             kPaperQuantiser);
}

int32_t int8_reduce_chunk_static(const uint8_t* const* peer_codes, const float* const* peer_luts, uint32_t W,
                                 const float* local_fp32, uint32_t divisor, uint64_t n,
                                 const uint64_t* seg_offsets, uint32_t T, float* acc_out, uint8_t* codes_out,
                                 float* lut_out, diloco_qparams* qparams_out, void* stream) {
    if (T > DILOCO_STATIC_MAX_SEGMENTS) return DILOCO_ERR_STATIC_LIMIT;
    void* ws = nullptr;
    int32_t rc = static_scratch(&ws);
    if (rc) return rc;
    return reduce_chunk_impl(peer_codes, peer_luts, W, local_fp32, divisor, n, seg_offsets, T, acc_out, codes_out,
                             lut_out, qparams_out, ws, kStaticScratchBytes, (hipStream_t)stream, kPaperQuantiser);
}

int32_t int8_reduce_chunk_variant(const uint8_t* const* peer_codes, const float* const* peer_luts, uint32_t W,
                                  const float* local_fp32, uint32_t divisor, uint64_t n,
                                  const uint64_t* seg_offsets, uint32_t T, float* acc_out, uint8_t* codes_out,
                                  float* lut_out, diloco_qparams* qparams_out, void* workspace,
                                  size_t workspace_bytes, void* stream, double range_sigmas, uint32_t codebook) {
    int32_t rc = check_variant(range_sigmas, codebook);
    if (rc) return rc;
    return reduce_chunk_impl(peer_codes, peer_luts, W, local_fp32, divisor, n, seg_offsets, T, acc_out, codes_out,
                             lut_out, qparams_out, workspace, workspace_bytes, (hipStream_t)stream,
                             QuantVariant{range_sigmas, codebook});
}

int32_t outer_nesterov_step(float* theta_outer, float* momentum, const float* delta_fp32,
                            const uint8_t* delta_codes, const float* delta_lut, const uint64_t* seg_offsets,
                            uint32_t T, uint64_t N, float lr, float beta, void* theta_local_out,
                            int32_t local_dtype, void* workspace, size_t workspace_bytes, void* stream_) {
    hipStream_t stream = (hipStream_t)stream_;
    const bool coded = delta_codes != nullptr || delta_lut != nullptr;
    if (coded == (delta_fp32 != nullptr)) return DILOCO_ERR_NULL;       // exactly one form
    if (coded && (!delta_codes || !delta_lut)) return DILOCO_ERR_NULL;
    if (N > 0 && (!theta_outer || !momentum)) return DILOCO_ERR_NULL;
    if (theta_local_out && local_dtype != DILOCO_DTYPE_FP32 && local_dtype != DILOCO_DTYPE_BF16)
        return DILOCO_ERR_DTYPE;
    if (misaligned(theta_outer, 4) || misaligned(momentum, 4) || misaligned(delta_fp32, 4) ||
        misaligned(delta_lut, 4) ||
        misaligned(theta_local_out, local_dtype == DILOCO_DTYPE_BF16 ? 2 : 4))
        return DILOCO_ERR_ALIGN;
    const uint64_t* seg_dev = nullptr;
    unsigned long long* counter = nullptr;
    if (coded) {
        int32_t rc = check_segments(seg_offsets, T, N);
        if (rc) return rc;
        if (!workspace) return DILOCO_ERR_NULL;
        if (misaligned(workspace, 256)) return DILOCO_ERR_ALIGN;
        const WorkspaceLayout L = workspace_layout(T);
        if (workspace_bytes < L.total) return DILOCO_ERR_WORKSPACE;
        if (N == 0) return DILOCO_OK;
        DILOCO_TRY(upload_offsets(seg_offsets, T + 1, (uint64_t*)((char*)workspace + L.seg), stream));
        seg_dev = (const uint64_t*)((char*)workspace + L.seg);
        counter = (unsigned long long*)((char*)workspace + L.counters) + 2;
    } else if (workspace) {
        // optional for the fp32 form: with a workspace the blocks claim chunks, without one each
        // block walks one static share
        if (misaligned(workspace, 256)) return DILOCO_ERR_ALIGN;
        const WorkspaceLayout L = workspace_layout(1);
        if (workspace_bytes < L.total) return DILOCO_ERR_WORKSPACE;
        counter = (unsigned long long*)((char*)workspace + L.counters) + 2;
    }
    if (N == 0) return DILOCO_OK;
    int cus = 0;
    int32_t rc = num_compute_units(&cus);
    if (rc) return rc;
    const int out = !theta_local_out ? kOutNone : (local_dtype == DILOCO_DTYPE_BF16 ? kOutBf16 : kOutF32);
    switch (out) {
        case kOutNone:
            DILOCO_TRY(run_outer<kOutNone>(theta_outer, momentum, delta_fp32, delta_codes, delta_lut, seg_dev,
                                           T, N, lr, beta, theta_local_out, cus, counter, stream));
            break;
        case kOutF32:
            DILOCO_TRY(run_outer<kOutF32>(theta_outer, momentum, delta_fp32, delta_codes, delta_lut, seg_dev,
                                          T, N, lr, beta, theta_local_out, cus, counter, stream));
            break;
        default:
            DILOCO_TRY(run_outer<kOutBf16>(theta_outer, momentum, delta_fp32, delta_codes, delta_lut, seg_dev,
                                           T, N, lr, beta, theta_local_out, cus, counter, stream));
            break;
    }
    return DILOCO_OK;
}

}  // extern "C"
