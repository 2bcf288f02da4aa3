// The small kernels around the two streaming passes: clearing the accumulators, turning a
// segment's sums into its quantisation range, and turning bucket sums into the codebook.
// Included by exactly one translation unit.
#pragma once

#include "device_common.h"

namespace diloco {

// Items 1-3 of Section 2.2: mean, sample standard deviation, range [mean - c std, mean + c std]
// (c = range_sigmas, 6 in the paper), 256 equal buckets; fp64 throughout, rounded once to the fp32
// pair the bucket index uses.
__global__ void finalize_qparams_kernel(const uint64_t* __restrict__ seg, uint32_t T,
                                        const double* __restrict__ stats,
                                        const float* __restrict__ pivot, double range_sigmas,
                                        diloco_qparams* __restrict__ qp) {
    uint32_t s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= T) return;
    diloco_qparams r;
    r.n = seg[s + 1] - seg[s];
    r.mean = 0.0;
    r.std = 0.0;
    r.lo = 0.0f;
    r.inv_w = 0.0f;
    r.status = 0;
    r.pad = 0;
    if (r.n == 0) {
        r.status = DILOCO_STATUS_EMPTY;
        qp[s] = r;
        return;
    }
    const double n = (double)r.n;
    const double s1 = stats[2 * (size_t)s], s2 = stats[2 * (size_t)s + 1];
    const double mean = (double)pivot[s] + s1 / n;
    double var = 0.0;
    if (r.n > 1) {
        var = (s2 - s1 * (s1 / n)) / (n - 1.0);
        if (var < 0.0) var = 0.0;
    }
    const double sd = sqrt(var);
    r.mean = mean;
    r.std = sd;
    if (!isfinite(mean) || !isfinite(sd)) r.status |= DILOCO_STATUS_NONFINITE;
    const double lo64 = mean - range_sigmas * sd;
    const double w64 = (2.0 * range_sigmas * sd) / 256.0;
    r.lo = (float)lo64;
    if (sd > 0.0) {
        float cand = (float)(1.0 / w64);
        if (isfinite(cand)) r.inv_w = cand;
    }
    if (r.inv_w == 0.0f) r.status |= DILOCO_STATUS_DEGENERATE;
    qp[s] = r;
}

// Item 4 of Section 2.2: codebook entry = average of the values in the bucket.  The bins hold
// integer sums of scaled offsets from the bucket centre (plus, for buckets 0 and 255, fp64 sums of
// the far clipped values), so the average offset is rebuilt in fp64 and the centre added back.
// An empty bucket gets its midpoint; with the midpoint codebook every bucket does.
__global__ __launch_bounds__(kThreads) void finalize_lut_kernel(uint32_t T, double range_sigmas,
                                                               uint32_t codebook,
                                                               const diloco_qparams* __restrict__ qp,
                                                               const unsigned long long* __restrict__ hsumq,
                                                               const unsigned long long* __restrict__ hcnt,
                                                               const double* __restrict__ osum,
                                                               const unsigned long long* __restrict__ ocnt,
                                                               float* __restrict__ lut) {
    const uint32_t s = blockIdx.x;
    const int k = threadIdx.x;
    if (s >= T) return;
    const diloco_qparams q = qp[s];
    unsigned long long c = hcnt[(size_t)s * kBuckets + k];
    const float w = bucket_width(q.inv_w);
    const float scale = offset_scale(q.inv_w);
    double off_sum = scale > 0.0f ? (double)(long long)hsumq[(size_t)s * kBuckets + k] / (double)scale : 0.0;
    if (k == 0 || k == kBuckets - 1) {
        const int e = k == 0 ? 0 : 1;
        c += ocnt[2 * (size_t)s + e];
        off_sum += osum[2 * (size_t)s + e];
    }
    float out;
    if (c > 0 && codebook == DILOCO_CODEBOOK_MEAN) {
        out = (float)((double)bucket_centre((float)k, bucket_centre0(q.lo, w), w) + off_sum / (double)c);
    } else {
        const double lo64 = q.mean - range_sigmas * q.std;
        const double w64 = (2.0 * range_sigmas * q.std) / 256.0;
        out = (float)(lo64 + ((double)k + 0.5) * w64);
    }
    lut[(size_t)s * kBuckets + k] = out;
}

__global__ void zero_kernel(uint64_t* p, size_t n_words) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n_words; i += stride) p[i] = 0;
}

}  // namespace diloco
