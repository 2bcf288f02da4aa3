/*
 * CPU oracle for the DiLoCo outer-synchronisation arithmetic of the INTELLECT-1 / PRIME
 * technical report (arXiv 2412.01152).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain definition that the GPU library is
 * checked against.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may call
 * it; the product path never does.  It shares no code, header, table or helper with the GPU path.
 *
 * What it computes, and where the paper defines it:
 *   - pseudo-gradient  d = theta_outer - theta_local            (Algorithm 1, "averaging outer
 *                                                                gradients" line: theta^(t-1) - theta_i^(t))
 *   - quantiser Q      per-tensor mean/std, range [mu-6s, mu+6s], 256 equal buckets,
 *                      codebook = mean of the values that fall in each bucket
 *                                                               (Section 2.2, the four-item list)
 *   - reduce           dequantise every contribution, add in fp32, average, quantise again
 *                                                               (Section 2.2: reduction in full
 *                                                                precision, quantised only in transit;
 *                                                                Algorithm 1: the 1/k average)
 *   - outer step       SGD with Nesterov momentum on theta_outer (Section 2 intro; Algorithm 1
 *                                                                "outer optimization" line;
 *                                                                Table "Model Configuration": lr 0.7,
 *                                                                momentum 0.9)
 *
 * Readings taken where the paper is silent (each is a single constant or branch below):
 *   sample standard deviation (n-1);  floor bucket rule with clipping into buckets 0 and 255;
 *   unsigned byte codes;  clipped values count towards the end buckets' means;  an empty bucket
 *   gets its midpoint;  sigma == 0 gives all codes 0 and lut[0] = mean;  the 1/k division happens
 *   before requantising;  Nesterov in the form  m' = beta*m + g,  theta' = theta - lr*(g + beta*m').
 *
 * Precision: statistics in fp64 (their running sums in long double), bucket sums in fp64, plain
 * sequential loops in index order.  The bucket index is taken in fp32 as two separately rounded operations (subtract, multiply) because
 * the deployed quantiser works on fp32 tensors; the C compiler must not fuse them
 * (build with -ffp-contract=off).  OpenMP is used only across independent segments or independent
 * elements, so results do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_STATUS_DEGENERATE 1u
#define ORACLE_STATUS_NONFINITE 2u
#define ORACLE_STATUS_EMPTY 4u

#define ORACLE_NUM_BUCKETS 256
/* The paper's quantiser has range_sigmas = 6 and the bucket-mean codebook (midpoint_codebook = 0).
 * Both are arguments so that the variants the paper only argues about qualitatively (Section 2.2:
 * why clip, why a codebook of bucket means) can be measured: another clipping width, and a codebook
 * of bucket midpoints.  Every caller that reproduces the paper passes 6.0 and 0. */

typedef struct {
    double mean;     /* mu of the segment (fp64) */
    double std;      /* sigma of the segment, sample form (fp64) */
    float lo;        /* lower edge of the range, mu - 6 sigma, rounded to fp32 */
    float inv_w;     /* 1 / bucket width, rounded to fp32; 0 when degenerate */
    uint64_t n;      /* number of elements */
    uint32_t status; /* ORACLE_STATUS_* bits */
    uint32_t pad;
} oracle_qparams;

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int t) {
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

/* bf16 is the upper half of an fp32 bit pattern: widening is exact. */
static float bf16_to_f32(uint16_t h) {
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

/* fp32 -> bf16, round to nearest, ties to even; NaN stays NaN. */
static uint16_t f32_to_bf16(float f) {
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    if ((bits & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((bits >> 16) | 0x0040u);
    uint32_t keep_lsb = (bits >> 16) & 1u;
    bits += 0x7fffu + keep_lsb;
    return (uint16_t)(bits >> 16);
}

/* Algorithm 1, outer-gradient line: d_i = theta_outer_i - theta_local_i, one fp32 subtraction.
 * theta_local may be stored as bf16 (local_is_bf16 != 0); it is widened exactly first. */
void oracle_pseudograd(const float* theta_outer, const void* theta_local, int local_is_bf16,
                       uint64_t n, float* d) {
    const float* lf = (const float*)theta_local;
    const uint16_t* lh = (const uint16_t*)theta_local;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        float local = local_is_bf16 ? bf16_to_f32(lh[i]) : lf[i];
        d[i] = theta_outer[i] - local;
    }
}

/* Section 2.2, quantisation list, on one tensor x[0..n).
 * Writes codes[n], lut[256] and the statistics record. */
void oracle_quantize(const float* x, uint64_t n, double range_sigmas, int midpoint_codebook,
                     uint8_t* codes, float* lut, oracle_qparams* qp) {
    oracle_qparams r;
    memset(&r, 0, sizeof r);
    r.n = n;
    if (n == 0) {
        r.status = ORACLE_STATUS_EMPTY;
        for (int k = 0; k < ORACLE_NUM_BUCKETS; ++k) lut[k] = 0.0f;
        *qp = r;
        return;
    }

    /* item 1: mean and standard deviation of the tensor, two passes as the definition reads.
     * The two running sums are kept in long double (64-bit significand on x86): a sequential fp64
     * sum of n terms drifts by about sqrt(n) * 1e-16 * |mean|, which for a tensor whose mean is
     * thousands of standard deviations would be visible at the 1e-9 * sigma level the parity
     * tests hold the mean to.  The results are rounded to fp64 once. */
    long double sum = 0.0L;
    for (uint64_t i = 0; i < n; ++i) sum += (long double)x[i];
    double mu = (double)(sum / (long double)n);
    long double sq = 0.0L;
    for (uint64_t i = 0; i < n; ++i) {
        long double c = (long double)x[i] - (long double)mu;
        sq += c * c;
    }
    double sigma = (n > 1) ? (double)sqrtl(sq / (long double)(n - 1)) : 0.0;
    r.mean = mu;
    r.std = sigma;
    if (!isfinite(mu) || !isfinite(sigma)) r.status |= ORACLE_STATUS_NONFINITE;

    /* items 2 and 3: range [mu - 6 sigma, mu + 6 sigma] cut into 256 equal buckets */
    double lo64 = mu - range_sigmas * sigma;
    double w64 = (2.0 * range_sigmas * sigma) / (double)ORACLE_NUM_BUCKETS;
    float lo = (float)lo64;
    float inv_w = 0.0f;
    if (sigma > 0.0) {
        float cand = (float)(1.0 / w64);
        if (isfinite(cand)) inv_w = cand;
    }
    if (inv_w == 0.0f) r.status |= ORACLE_STATUS_DEGENERATE;
    r.lo = lo;
    r.inv_w = inv_w;

    /* bucket of every value (floor, clipped at both ends) and, item 4, the per-bucket sums */
    double bsum[ORACLE_NUM_BUCKETS];
    uint64_t bcnt[ORACLE_NUM_BUCKETS];
    for (int k = 0; k < ORACLE_NUM_BUCKETS; ++k) {
        bsum[k] = 0.0;
        bcnt[k] = 0;
    }
    for (uint64_t i = 0; i < n; ++i) {
        float u = x[i] - lo;
        float t = u * inv_w;
        int k;
        if (!(t > 0.0f))
            k = 0;
        else if (t >= 255.0f)
            k = 255;
        else
            k = (int)t;
        codes[i] = (uint8_t)k;
        bsum[k] += (double)x[i];
        bcnt[k] += 1;
    }
    for (int k = 0; k < ORACLE_NUM_BUCKETS; ++k) {
        if (bcnt[k] > 0 && !midpoint_codebook)
            lut[k] = (float)(bsum[k] / (double)bcnt[k]);
        else
            lut[k] = (float)(lo64 + ((double)k + 0.5) * w64);
    }
    *qp = r;
}

/* Decoding: x_hat_i = lut[code_i]. */
void oracle_dequantize(const uint8_t* codes, const float* lut, uint64_t n, float* out) {
    for (uint64_t i = 0; i < n; ++i) out[i] = lut[codes[i]];
}

/* Q applied segment by segment: segment s covers [seg_offsets[s], seg_offsets[s+1]).
 * luts is [T][256], qps is [T]. */
void oracle_quantize_segments(const float* x, const uint64_t* seg_offsets, uint32_t T,
                              double range_sigmas, int midpoint_codebook, uint8_t* codes,
                              float* luts, oracle_qparams* qps) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t s = 0; s < (int32_t)T; ++s) {
        uint64_t a = seg_offsets[s], b = seg_offsets[s + 1];
        oracle_quantize(x + a, b - a, range_sigmas, midpoint_codebook, codes + a,
                        luts + (size_t)s * ORACLE_NUM_BUCKETS, &qps[s]);
    }
}

/* Stage 1: pseudo-gradient, then Q per segment.  d_scratch is [N] fp32 scratch owned by the caller
 * (it holds the pseudo-gradient on return). */
void oracle_pseudograd_quantize(const float* theta_outer, const void* theta_local,
                                int local_is_bf16, uint64_t N, const uint64_t* seg_offsets,
                                uint32_t T, double range_sigmas, int midpoint_codebook,
                                float* d_scratch, uint8_t* codes, float* luts,
                                oracle_qparams* qps) {
    oracle_pseudograd(theta_outer, theta_local, local_is_bf16, N, d_scratch);
    oracle_quantize_segments(d_scratch, seg_offsets, T, range_sigmas, midpoint_codebook, codes, luts,
                             qps);
}

/* Stage 2: the local reduction step of the quantised all-reduce.
 * For every element: start from the un-quantised local addend (or 0), add each coded
 * contribution's decoded value in contribution order with one fp32 addition each, divide by
 * `divisor` (the k of Algorithm 1) in fp32, then quantise the result per segment.
 * peer_luts[p] is [T][256].  acc is [n] (required; receives the averaged fp32 values). */
void oracle_reduce(const uint8_t* const* peer_codes, const float* const* peer_luts, uint32_t W,
                   const float* local_fp32, uint32_t divisor, uint64_t n,
                   const uint64_t* seg_offsets, uint32_t T, double range_sigmas,
                   int midpoint_codebook, float* acc, uint8_t* codes_out, float* luts_out,
                   oracle_qparams* qps_out) {
    float fdiv = (float)divisor;
    (void)n; /* seg_offsets[T] == n */
    for (uint32_t s = 0; s < T; ++s) {
        uint64_t a = seg_offsets[s], b = seg_offsets[s + 1];
#pragma omp parallel for schedule(static)
        for (int64_t i = (int64_t)a; i < (int64_t)b; ++i) {
            float v = local_fp32 ? local_fp32[i] : 0.0f;
            for (uint32_t p = 0; p < W; ++p) {
                const float* lut = peer_luts[p] + (size_t)s * ORACLE_NUM_BUCKETS;
                v = v + lut[peer_codes[p][i]];
            }
            acc[i] = v / fdiv;
        }
    }
    oracle_quantize_segments(acc, seg_offsets, T, range_sigmas, midpoint_codebook, codes_out,
                             luts_out, qps_out);
}

/* Stage 3: outer optimiser, SGD with Nesterov momentum.
 *   g      = delta_fp32[i]                     (fp32 form), or
 *            delta_luts[s][delta_codes[i]]     (coded form, s = segment of i)
 *   m'     = beta * m + g
 *   theta' = theta - lr * (g + beta * m')
 * evaluated in fp64 from the fp32 inputs, each result rounded once to fp32.
 * theta_local_out (optional) receives theta' in fp32 (out_is_bf16 == 0) or bf16. */
void oracle_outer_step(float* theta, float* momentum, const float* delta_fp32,
                       const uint8_t* delta_codes, const float* delta_luts,
                       const uint64_t* seg_offsets, uint32_t T, uint64_t N, float lr, float beta,
                       void* theta_local_out, int out_is_bf16) {
    double lr64 = (double)lr, beta64 = (double)beta;
    if (delta_fp32) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < (int64_t)N; ++i) {
            double g = (double)delta_fp32[i];
            double m_new = beta64 * (double)momentum[i] + g;
            double th_new = (double)theta[i] - lr64 * (g + beta64 * m_new);
            momentum[i] = (float)m_new;
            theta[i] = (float)th_new;
        }
    } else {
        for (uint32_t s = 0; s < T; ++s) {
            const float* lut = delta_luts + (size_t)s * ORACLE_NUM_BUCKETS;
            uint64_t a = seg_offsets[s], b = seg_offsets[s + 1];
#pragma omp parallel for schedule(static)
            for (int64_t i = (int64_t)a; i < (int64_t)b; ++i) {
                double g = (double)lut[delta_codes[i]];
                double m_new = beta64 * (double)momentum[i] + g;
                double th_new = (double)theta[i] - lr64 * (g + beta64 * m_new);
                momentum[i] = (float)m_new;
                theta[i] = (float)th_new;
            }
        }
    }
    if (theta_local_out) {
        if (out_is_bf16) {
            uint16_t* o = (uint16_t*)theta_local_out;
#pragma omp parallel for schedule(static)
            for (int64_t i = 0; i < (int64_t)N; ++i) o[i] = f32_to_bf16(theta[i]);
        } else {
            float* o = (float*)theta_local_out;
#pragma omp parallel for schedule(static)
            for (int64_t i = 0; i < (int64_t)N; ++i) o[i] = theta[i];
        }
    }
}
