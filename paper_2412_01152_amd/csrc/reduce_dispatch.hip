// Stage 2 kernels for one group of W values (number of coded contributions), selected at compile
// time with -DDILOCO_W_GROUP=0..3 : W in {0..4}, {5..8}, {9..12}, {13..16}.  W is a template
// argument so that all W code-stream loads of an iteration are in flight together and the W
// codebooks sit at fixed LDS offsets.
#include <algorithm>

#include "kernels.h"
#include "launch.h"

#ifndef DILOCO_W_GROUP
#error "compile with -DDILOCO_W_GROUP=0..3"
#endif

namespace diloco {
namespace {

template <int W, bool kLocal, bool kTrueDiv>
SrcReduce<W, kLocal, kTrueDiv> make_src(const ReduceArgs& a) {
    SrcReduce<W, kLocal, kTrueDiv> s;
    for (int p = 0; p < SrcReduce<W, kLocal, kTrueDiv>::kW; ++p) {
        s.codes[p] = p < W ? a.codes[p] : nullptr;
        s.luts[p] = p < W ? a.luts[p] : nullptr;
    }
    s.local = a.local;
    s.div = a.div;
    s.lds = nullptr;
    return s;
}

template <int W, bool kLocal, bool kTrueDiv, bool kWriteAcc>
hipError_t run_stats(const ReduceArgs& a, const Pass& p, float* acc_out) {
    using Src = SrcReduce<W, kLocal, kTrueDiv>;
    hipLaunchKernelGGL(pivot_kernel<Src>, dim3((p.T + kPivotSegmentsPerBlock - 1) / kPivotSegmentsPerBlock),
                       dim3(kThreads), 0, p.stream,
                       make_src<W, kLocal, kTrueDiv>(a), p.seg, p.T, p.pivot);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr auto kernel = stats_kernel<Src, kWriteAcc>;
    const uint32_t phase = acc_out ? host_phase(acc_out, 4)
                                   : (W > 0 ? host_phase(a.codes[0], 1) : host_phase(a.local, 4));
    int bpc = resident_blocks_per_cu<kernel>();
    if (kWriteAcc) bpc = std::min(bpc, blocks_per_cu_store_acc(W));
    Grid g = plan_grid(p.N, p.num_cus, bpc, p.counters + 0, phase,
                       kWriteAcc ? chunk_iters_store_acc(W, kLocal) : kChunkItersRead);
    (void)mark(0, p.stream);
    hipLaunchKernelGGL(kernel, dim3(g.blocks), dim3(kThreads), 0, p.stream, make_src<W, kLocal, kTrueDiv>(a), p.seg,
                       p.T, p.N, g.work, p.stats, p.pivot, acc_out);
    e = hipGetLastError();
    (void)mark(1, p.stream);
    return e;
}

template <int W, bool kLocal, bool kTrueDiv, int kCopies>
hipError_t run_quant_as(const ReduceArgs& a, const Pass& p, const diloco_qparams* qp, uint8_t* codes) {
    using Src = SrcReduce<W, kLocal, kTrueDiv>;
    constexpr auto kernel = quant_kernel<Src, kCopies, Src::kStage>;
    // with bins the look-ups and LDS atomics need every wave that fits; without them the memory side
    // decides, and it prefers fewer blocks and shorter chunks (a narrower window of active addresses)
    const int bpc = kCopies > 0 ? resident_blocks_per_cu<kernel>()
                                : std::min(resident_blocks_per_cu<kernel>(), kBlocksPerCuReduceNoBins);
    Grid g = plan_grid(p.N, p.num_cus, bpc, p.counters + 1, host_phase(codes, 1),
                       kCopies > 0 ? kChunkItersReduceWrite : kChunkItersReduceNoBins);
    (void)mark(2, p.stream);
    hipLaunchKernelGGL(kernel, dim3(g.blocks), dim3(kThreads), 0, p.stream, make_src<W, kLocal, kTrueDiv>(a), p.seg,
                       p.T, p.N, g.work, qp, codes, PassBOut{p.hsumq, p.hcnt, p.osum, p.ocnt}, p.write_phase);
    hipError_t e = hipGetLastError();
    (void)mark(3, p.stream);
    return e;
}

template <int W, bool kLocal, bool kTrueDiv>
hipError_t run_quant(const ReduceArgs& a, const Pass& p, const diloco_qparams* qp, uint8_t* codes) {
    return p.bins ? run_quant_as<W, kLocal, kTrueDiv, kBinCopiesReduce>(a, p, qp, codes)
                  : run_quant_as<W, kLocal, kTrueDiv, 0>(a, p, qp, codes);
}

template <int W, bool kLocal, bool kTrueDiv>
hipError_t stats_wld(const ReduceArgs& a, const Pass& p, float* acc_out) {
    return acc_out ? run_stats<W, kLocal, kTrueDiv, true>(a, p, acc_out)
                   : run_stats<W, kLocal, kTrueDiv, false>(a, p, acc_out);
}

template <int W>
hipError_t stats_w(const ReduceArgs& a, const Pass& p, float* acc_out) {
    if (a.local)
        return a.true_div ? stats_wld<W, true, true>(a, p, acc_out) : stats_wld<W, true, false>(a, p, acc_out);
    if constexpr (W == 0)
        return hipErrorInvalidValue;
    else
        return a.true_div ? stats_wld<W, false, true>(a, p, acc_out) : stats_wld<W, false, false>(a, p, acc_out);
}

template <int W>
hipError_t quant_w(const ReduceArgs& a, const Pass& p, const diloco_qparams* qp, uint8_t* codes) {
    if (a.local)
        return a.true_div ? run_quant<W, true, true>(a, p, qp, codes) : run_quant<W, true, false>(a, p, qp, codes);
    if constexpr (W == 0)
        return hipErrorInvalidValue;
    else
        return a.true_div ? run_quant<W, false, true>(a, p, qp, codes)
                          : run_quant<W, false, false>(a, p, qp, codes);
}

}  // namespace

#define DILOCO_CAT2(a, b) a##b
#define DILOCO_CAT(a, b) DILOCO_CAT2(a, b)
#define DILOCO_STATS_FN DILOCO_CAT(launch_reduce_stats_g, DILOCO_W_GROUP)
#define DILOCO_QUANT_FN DILOCO_CAT(launch_reduce_quant_g, DILOCO_W_GROUP)

#if DILOCO_W_GROUP == 0
#define DILOCO_W0 0
#else
#define DILOCO_W0 (DILOCO_W_GROUP * 4 + 1)
#endif

hipError_t DILOCO_STATS_FN(const ReduceArgs& a, const Pass& p, float* acc_out) {
    switch ((int)a.W - DILOCO_W0) {
        case 0: return stats_w<DILOCO_W0 + 0>(a, p, acc_out);
        case 1: return stats_w<DILOCO_W0 + 1>(a, p, acc_out);
        case 2: return stats_w<DILOCO_W0 + 2>(a, p, acc_out);
        case 3: return stats_w<DILOCO_W0 + 3>(a, p, acc_out);
#if DILOCO_W_GROUP == 0
        case 4: return stats_w<4>(a, p, acc_out);
#endif
        default: return hipErrorInvalidValue;
    }
}

hipError_t DILOCO_QUANT_FN(const ReduceArgs& a, const Pass& p, const diloco_qparams* qp, uint8_t* codes) {
    switch ((int)a.W - DILOCO_W0) {
        case 0: return quant_w<DILOCO_W0 + 0>(a, p, qp, codes);
        case 1: return quant_w<DILOCO_W0 + 1>(a, p, qp, codes);
        case 2: return quant_w<DILOCO_W0 + 2>(a, p, qp, codes);
        case 3: return quant_w<DILOCO_W0 + 3>(a, p, qp, codes);
#if DILOCO_W_GROUP == 0
        case 4: return quant_w<4>(a, p, qp, codes);
#endif
        default: return hipErrorInvalidValue;
    }
}

}  // namespace diloco
