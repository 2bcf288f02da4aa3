/*
 * diloco_mi355 - the DiLoCo outer-synchronisation arithmetic on one AMD MI355X (gfx950).
 *
 * C ABI of the library built from paper_2412_01152_amd/csrc/.  The three operations are the
 * compute that one device performs on its share of the model at every outer step of DiLoCo as
 * described in the INTELLECT-1 technical report (arXiv 2412.01152):
 *
 *   diloco_pseudograd_quantize   Algorithm 1, outer-gradient line (theta^(t-1) - theta_i^(t)),
 *                                followed by the 8-bit quantiser of Section 2.2 (four-item list)
 *   int8_reduce_chunk            Section 2.2: the reduce step of the quantised all-reduce, done in
 *                                fp32 on decoded values, averaged (the 1/k of Algorithm 1) and
 *                                quantised again for transmission
 *   outer_nesterov_step          Algorithm 1, outer-optimisation line, with SGD + Nesterov momentum
 *                                (Section 2 intro; Appendix "Model Configuration": lr 0.7, mu 0.9)
 *
 * General conventions
 *   - "device" pointers are HIP device memory on the current device; "host" pointers are ordinary
 *     host memory.  All buffers are owned by the caller.  The library allocates and frees nothing
 *     and never synchronises the device.
 *   - Every call only enqueues work on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream) and returns.  Host arrays (seg_offsets, pointer tables) are consumed before the call
 *     returns and may be reused at once.  What is enqueued is kernels only - no copies, no memset
 *     nodes, no events unless diloco_profile_passes asked for them - so the calls may be recorded
 *     by a stream capture and replayed as a HIP graph (segment offsets and pointer tables are
 *     frozen into the recording).
 *   - A flat buffer of N elements is cut into T contiguous "segments" (the paper's "tensors":
 *     the quantisation groups).  `seg_offsets` is a HOST array of T+1 ascending element offsets
 *     with seg_offsets[0] == 0 and seg_offsets[T] == N.  Empty segments are allowed.
 *   - Codes are one unsigned byte per element (bucket index 0..255).  A codebook ("lut") is 256
 *     fp32 values per segment: luts are [T][256], row-major.
 *   - Pointers need only their natural alignment (4 bytes for fp32, 2 for bf16, 1 for codes,
 *     8 for diloco_qparams, 256 for the workspace); 16-byte aligned buffers run fastest.
 *   - Return value: 0 on success; a negative DILOCO_ERR_* for an argument error found on the host
 *     (nothing has been enqueued); a positive value is the hipError_t of a failed launch.
 *     Data-dependent conditions (constant tensor, NaN input, empty segment) never fail a call:
 *     they are reported per segment in diloco_qparams.status.
 *   - Calls that use the same workspace must be ordered on one stream.
 *   - State.  The library keeps no data between calls: every result is a function of the call's
 *     arguments.  What it does keep, per process, is (a) the number of resident blocks per compute
 *     unit of each kernel, looked up once (thread-safe), and (b) two instrumentation settings that
 *     only the calls at the end of this header change and that never alter results:
 *     diloco_profile_passes (per host thread) and diloco_tune_write_phase (per process).  No
 *     environment variable is read.
 *   - The second pass of diloco_pseudograd_quantize holds its output codes back in on-chip memory
 *     and writes them during a periodic window of the device's constant-rate clock (the first 10 us
 *     of every 40 us), which the memory system serves faster than a steady trickle of writes among
 *     the reads; buffers below 2^27 elements are written at once.
 */
#ifndef DILOCO_MI355_H
#define DILOCO_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DILOCO_DTYPE_FP32 0
#define DILOCO_DTYPE_BF16 1

#define DILOCO_MAX_PEERS 16u        /* largest W accepted by int8_reduce_chunk */
#define DILOCO_MAX_SEGMENTS 65536u  /* largest T accepted */
#define DILOCO_MAX_RING_NODES 20u   /* largest n accepted by diloco_ring_order */
#define DILOCO_STATIC_MAX_SEGMENTS 512u /* largest T accepted by int8_reduce_chunk_static */

#define DILOCO_OK 0
#define DILOCO_ERR_NULL (-1)        /* a required pointer is NULL                         */
#define DILOCO_ERR_SIZE (-2)        /* bad N / T / W / divisor / seg_offsets               */
#define DILOCO_ERR_ALIGN (-3)       /* a pointer is not aligned to its element type        */
#define DILOCO_ERR_WORKSPACE (-4)   /* workspace smaller than diloco_workspace_bytes(T)    */
#define DILOCO_ERR_DTYPE (-5)       /* unknown dtype flag                                  */
#define DILOCO_ERR_STATIC_LIMIT (-6) /* T above DILOCO_STATIC_MAX_SEGMENTS (int8_reduce_chunk_static) */

#define DILOCO_CODEBOOK_MEAN 0u      /* codebook entry = average of the bucket's values (the paper's) */
#define DILOCO_CODEBOOK_MIDPOINT 1u  /* codebook entry = centre of the bucket                         */
#define DILOCO_MIN_RANGE_SIGMAS 0.5  /* bounds on range_sigmas of the *_variant calls                 */
#define DILOCO_MAX_RANGE_SIGMAS 64.0

#define DILOCO_STATUS_DEGENERATE 1u /* sigma == 0 (or 1/width not finite): all codes 0, lut[0] = mean */
#define DILOCO_STATUS_NONFINITE 2u  /* NaN/Inf reached the statistics; codes unspecified            */
#define DILOCO_STATUS_EMPTY 4u      /* segment has no elements; lut is all zeros                     */

/* Per-segment record written by the two quantising calls (device memory, T records).
 * Section 2.2 items 1-3: mean and standard deviation (sample form, n-1) of the segment in fp64,
 * and the fp32 values the bucket index is computed with:
 *     lo    = fp32(mean - 6 std)               lower edge of the clipping range
 *     inv_w = fp32(256 / (12 std))             reciprocal of the bucket width (0 if degenerate)
 *     code  = clamp(floor((x - lo) * inv_w), 0, 255)   with the subtraction and the product each
 *                                                      rounded to fp32 */
typedef struct diloco_qparams {
    double mean;
    double std;
    float lo;
    float inv_w;
    uint64_t n;
    uint32_t status;
    uint32_t pad;
} diloco_qparams;

/* Bytes of device scratch the two quantising calls need for T segments (0 < T <= DILOCO_MAX_SEGMENTS). */
size_t diloco_workspace_bytes(uint32_t T);

/* Human-readable text for a return value of this library (static storage). */
const char* diloco_strerror(int32_t code);

/*
 * Stage 1.  For every element  d = theta_outer - widen(theta_local)  (one fp32 subtraction; bf16 is
 * widened exactly), then per segment the quantiser of Section 2.2:  mean/std of d, range
 * [mean - 6 std, mean + 6 std] in 256 equal buckets, values outside clipped into buckets 0 / 255,
 * codebook entry = average of the segment's values that fell into the bucket (empty bucket: its
 * midpoint).  d itself is never written to memory.
 *
 *   theta_outer  device, [N] fp32            the outer parameters theta^(t-1)
 *   theta_local  device, [N] fp32 or bf16    this worker's parameters after its inner steps
 *   local_dtype  DILOCO_DTYPE_FP32 / DILOCO_DTYPE_BF16 (dtype of theta_local)
 *   seg_offsets  host,   [T+1]
 *   codes_out    device, [N] bytes           out
 *   lut_out      device, [T][256] fp32       out
 *   qparams_out  device, [T]                 out
 *   workspace    device, >= diloco_workspace_bytes(T) bytes, 256-byte aligned; contents are
 *                scratch (overwritten by every call)
 * N == 0 is allowed (all segments empty).  Inputs are not modified; outputs must not overlap inputs.
 */
int32_t diloco_pseudograd_quantize(const float* theta_outer, const void* theta_local,
                                   int32_t local_dtype, uint64_t N, const uint64_t* seg_offsets,
                                   uint32_t T, uint8_t* codes_out, float* lut_out,
                                   diloco_qparams* qparams_out, void* workspace,
                                   size_t workspace_bytes, void* stream);

/*
 * Stage 2.  The local reduce step of the 8-bit all-reduce on a chunk of n elements (Section 2.2:
 * values are quantised only in transit, the reduction itself runs in fp32).  For every element
 *     v = local_fp32[i]            (0 if local_fp32 is NULL)
 *     v = v + peer_luts[p][s][peer_codes[p][i]]     for p = 0 .. W-1 in this order, one fp32
 *                                                   addition each (s = segment of i)
 *     a = v / divisor              fp32 division; divisor is the k of Algorithm 1's average
 * and then (codes_out, lut_out, qparams_out) = quantiser of Section 2.2 applied to a, per segment.
 *
 *   peer_codes   HOST array of W device pointers, each [n] bytes
 *   peer_luts    HOST array of W device pointers, each [T][256] fp32
 *   W            number of coded contributions, 0..DILOCO_MAX_PEERS; W + (local_fp32 != NULL) >= 1
 *   local_fp32   device, [n] fp32, optional un-quantised addend (the chunk owner's own data)
 *   divisor      >= 1; it is separate from W because joiners that contribute zeros and retries
 *                with fewer peers (Sections 2.4.2, 2.4.5) change one without the other
 *   seg_offsets  host, [T+1], offsets inside the chunk (T = 1: the chunk is one quantisation group)
 *   acc_out      device, [n] fp32, optional: receives a.  MAY be the same buffer as local_fp32.
 *                When given, a is stored once and read back for the second pass; when NULL, a is
 *                recomputed from the codes in the second pass.
 *   codes_out, lut_out, qparams_out, workspace: as in stage 1.  codes_out MAY be the same buffer as
 *                one of the peer_codes (every element's inputs are read before its code is
 *                written; that contribution is consumed).
 * The call is a pure function of its inputs: calling it again with a smaller W on the same
 * buffers is the retry of Section 2.4.5.
 */
int32_t int8_reduce_chunk(const uint8_t* const* peer_codes, const float* const* peer_luts,
                          uint32_t W, const float* local_fp32, uint32_t divisor, uint64_t n,
                          const uint64_t* seg_offsets, uint32_t T, float* acc_out,
                          uint8_t* codes_out, float* lut_out, diloco_qparams* qparams_out,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * int8_reduce_chunk for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error behaviour as int8_reduce_chunk, without `workspace` and
 * `workspace_bytes`: the scratch (segment offsets, fp64 sums, pivots, bucket bins, chunk counters) lives
 * in a device array that is part of the library's code object, about 2.1 MB
 * (= diloco_workspace_bytes(DILOCO_STATIC_MAX_SEGMENTS)), which every GPU the library runs on holds
 * until the process ends.
 *   - T > DILOCO_STATIC_MAX_SEGMENTS is refused with DILOCO_ERR_STATIC_LIMIT before anything is enqueued.
 *   - The call allocates and frees nothing, on the host or on the device.  The first call on a device
 *     looks up that device's address of the array (a symbol lookup, no allocation); make that first
 *     call outside a stream capture.
 *   - Every call on a GPU uses that GPU's one array (the call clears what must start at zero, on the
 *     stream): calls on the same GPU must not overlap in time - order them on one stream, or with
 *     events - or they race on the scratch.  Calls that pass their own workspace are unaffected.
 */
int32_t int8_reduce_chunk_static(const uint8_t* const* peer_codes, const float* const* peer_luts,
                                 uint32_t W, const float* local_fp32, uint32_t divisor, uint64_t n,
                                 const uint64_t* seg_offsets, uint32_t T, float* acc_out,
                                 uint8_t* codes_out, float* lut_out, diloco_qparams* qparams_out,
                                 void* stream);

/*
 * The two quantising calls with the quantiser's two constants as arguments.  Section 2.2 fixes a
 * clipping range of +-6 standard deviations and a codebook of bucket averages, and argues for both
 * only in words (outliers are clipped to keep the buckets narrow; averages instead of centres lower
 * the error); these calls let the alternatives be measured on the same kernels.
 *     range_sigmas   half-width c of the range [mean - c std, mean + c std], in
 *                    [DILOCO_MIN_RANGE_SIGMAS, DILOCO_MAX_RANGE_SIGMAS] (else DILOCO_ERR_SIZE);
 *                    lo = fp32(mean - c std), inv_w = fp32(256 / (2 c std))
 *     codebook       DILOCO_CODEBOOK_MEAN or DILOCO_CODEBOOK_MIDPOINT (else DILOCO_ERR_DTYPE); with
 *                    MIDPOINT lut[k] = fp32(mean - c std + (k + 1/2) * 2 c std / 256) for every k,
 *                    clipped values included
 * With range_sigmas = 6.0 and DILOCO_CODEBOOK_MEAN they are the calls above, bit for bit.  All other
 * arguments, layouts and error behaviour are those of the calls above.
 */
int32_t diloco_pseudograd_quantize_variant(const float* theta_outer, const void* theta_local,
                                           int32_t local_dtype, uint64_t N,
                                           const uint64_t* seg_offsets, uint32_t T, uint8_t* codes_out,
                                           float* lut_out, diloco_qparams* qparams_out,
                                           void* workspace, size_t workspace_bytes, void* stream,
                                           double range_sigmas, uint32_t codebook);
int32_t int8_reduce_chunk_variant(const uint8_t* const* peer_codes, const float* const* peer_luts,
                                  uint32_t W, const float* local_fp32, uint32_t divisor, uint64_t n,
                                  const uint64_t* seg_offsets, uint32_t T, float* acc_out,
                                  uint8_t* codes_out, float* lut_out, diloco_qparams* qparams_out,
                                  void* workspace, size_t workspace_bytes, void* stream,
                                  double range_sigmas, uint32_t codebook);

/*
 * Stage 3.  Outer optimiser step, SGD with Nesterov momentum (Algorithm 1, outer-optimisation
 * line), in place:
 *     g      = delta_fp32[i]                              (fp32 form), or
 *              delta_lut[s][delta_codes[i]]               (coded form: what every replica receives
 *                                                          from the all-gather; s = segment of i)
 *     m'     = beta * m + g
 *     theta' = theta - lr * (g + beta * m')
 * in fp32 (fused multiply-adds allowed).
 *
 *   theta_outer  device, [N] fp32, in/out
 *   momentum     device, [N] fp32, in/out (zero it before the first outer step)
 *   delta_fp32   device, [N] fp32, or NULL       exactly one of delta_fp32 and
 *   delta_codes  device, [N] bytes, or NULL      (delta_codes, delta_lut) must be given
 *   delta_lut    device, [T][256] fp32, or NULL
 *   seg_offsets  host, [T+1]; used by the coded form only (may be NULL with T = 0 otherwise)
 *   lr, beta     the paper uses 0.7 and 0.9
 *   theta_local_out  device, [N] fp32 or bf16 (round to nearest even), optional: the new worker
 *                weights, i.e. a copy of theta' (steps 3-4 of Section 2.1's procedure).  In fp32 it
 *                MAY be the same buffer as delta_fp32 (the average is consumed).
 *   local_dtype  dtype of theta_local_out
 *   workspace    device, 256-byte aligned; required by the coded form (>= diloco_workspace_bytes(T)
 *                bytes); optional for the fp32 form (>= diloco_workspace_bytes(1) bytes, or NULL:
 *                the result is the same, the call is 1-3 % slower without one)
 */
int32_t outer_nesterov_step(float* theta_outer, float* momentum, const float* delta_fp32,
                            const uint8_t* delta_codes, const float* delta_lut,
                            const uint64_t* seg_offsets, uint32_t T, uint64_t N, float lr,
                            float beta, void* theta_local_out, int32_t local_dtype,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * Bandwidth-aware ring order (Section 2.5).  Given the measured bandwidth of every directed link,
 * finds an order of the n nodes, closed into a ring, whose slowest link is as fast as possible:
 * the Hamiltonian cycle C maximising min over its edges (u, v) of w(u, v).  Exact (threshold search
 * over the edge weights with a subset recurrence for Hamiltonicity), host code only, no device use.
 *
 *   bandwidth       HOST, [n][n] row-major doubles; bandwidth[u * n + v] is the rate from node u to
 *                   node v (any unit), finite and >= 0; the diagonal is ignored.  A symmetric
 *                   matrix describes undirected links.
 *   n               1 .. DILOCO_MAX_RING_NODES
 *   order_out       HOST, [n]: the ring order[0] -> order[1] -> ... -> order[n-1] -> order[0];
 *                   order[0] is node 0.  When several rings share the best bottleneck, any one of
 *                   them is returned.
 *   bottleneck_out  HOST, optional: the bandwidth of the slowest link of that ring (+infinity for n = 1)
 * Returns DILOCO_OK, DILOCO_ERR_NULL, or DILOCO_ERR_SIZE (n out of range, a negative or non-finite
 * bandwidth).
 */
int32_t diloco_ring_order(const double* bandwidth, uint32_t n, uint32_t* order_out,
                          double* bottleneck_out);

/*
 * Placement advice for callers that own one large device allocation (host arithmetic only).
 * On an MI355X the streaming kernels run 2 to 8 % faster when a buffer that a kernel WRITES does not lie
 * within about 64 GiB of the buffers the same kernel reads or updates (measured; it does not depend on the
 * low address bits).  Buffers of a few GiB that an allocator hands out one after the other all lie side by
 * side, which is the slow case; buffers of tens of GiB are far apart by themselves.  This call returns, for
 * an arena of arena_bytes, the byte offsets at which to start carving three groups of buffers:
 *     offsets_out[0]  "read"   what the three calls only read, or update in place while reading:
 *                              theta_outer, theta_local, the peers' codes
 *     offsets_out[1]  "state"  momentum, and the codes that diloco_pseudograd_quantize writes
 *     offsets_out[2]  "out"    the codes that int8_reduce_chunk writes (and outer_nesterov_step reads)
 * The groups start 100 GiB apart when the arena has room for that (216 GiB or more), else a third of
 * the arena apart; offsets are multiples of 4096.  Results never depend on placement.
 *   offsets_out  HOST, [3]
 * Returns DILOCO_OK, DILOCO_ERR_NULL, or DILOCO_ERR_SIZE (an arena below 12 KiB).
 */
int32_t diloco_placement(uint64_t arena_bytes, uint64_t* offsets_out);

/*
 * Instrumentation for benchmarks (not part of the method).  After this call, every later call of
 * the three operations made from the same host thread records HIP events on its stream around its
 * streaming kernels, so a harness can time each kernel without a profiler:
 *     events[0], events[1]   before / after the first streaming pass  (statistics pass of the two
 *                            quantising calls; the only pass of outer_nesterov_step)
 *     events[2], events[3]   before / after the second streaming pass (bucketise + codebook sums);
 *                            not recorded by outer_nesterov_step
 *   events   HOST array of 4 hipEvent_t created by the caller with timing enabled, or NULL to stop
 *            recording.  The array is copied; the events stay owned by the caller and must outlive
 *            the calls that record them.
 * Returns DILOCO_OK.
 */
int32_t diloco_profile_passes(void* const* events);

/*
 * Instrumentation for tests and benchmarks (not part of the method): when the second pass of
 * diloco_pseudograd_quantize writes the codes it holds back on chip.  Process-wide; applies to calls
 * made after it returns.  Results never depend on it.
 *     period_us < 0              the built-in choice (by buffer size, see the conventions above)
 *     period_us == 0             write every iteration's codes at once, at every size
 *     period_us > 0              hold codes back at EVERY size and write them during the first
 *                                window_us of every period_us microseconds (or when the on-chip
 *                                staging area is full); 1 <= window_us <= period_us <= 1,000,000
 * Returns DILOCO_OK, or DILOCO_ERR_SIZE for a window or period outside those bounds (nothing changes).
 */
int32_t diloco_tune_write_phase(int32_t period_us, int32_t window_us);

#ifdef __cplusplus
}
#endif
#endif /* DILOCO_MI355_H */
