/*
 * One outer synchronisation through the C ABI, from plain C: no Python, no torch.
 *
 *   stage 1  every worker's pseudo-gradient theta_outer - theta_local is quantised
 *            (Algorithm 1, outer-gradient line; Section 2.2's quantiser)
 *   stage 2  the W coded contributions are decoded, averaged in fp32 and quantised again
 *            (Section 2.2, the reduce step of the quantised all-reduce)
 *   stage 3  the outer Nesterov step is taken from the coded average
 *            (Algorithm 1, outer-optimisation line; lr 0.7, momentum 0.9)
 *
 * The program then checks on the host what the definitions fix exactly: the statistics, every bucket
 * index given the returned range (two fp32 operations, floor, clamp), the decoded fp32 sums in
 * contribution order, and the update rule.  It prints one line and returns 0 when all of it holds.
 * Built by `python -m paper_2412_01152_amd.build` next to the library.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/diloco_mi355.h"

#define W 3
#define T 3

#define HIP_OK(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));             \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)
#define LIB_OK(call)                                                                      \
    do {                                                                                  \
        int32_t rc_ = (call);                                                             \
        if (rc_ != 0) {                                                                   \
            fprintf(stderr, "%s failed: %d (%s)\n", #call, rc_, diloco_strerror(rc_));    \
            return 3;                                                                     \
        }                                                                                 \
    } while (0)

static uint64_t rng_state = 0x2412011520ull;
static double uniform(void) { /* splitmix64 -> (0, 1) */
    uint64_t z = (rng_state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    z ^= z >> 31;
    return ((double)(z >> 11) + 0.5) / 9007199254740992.0;
}
static double bell(void) { /* sum of 12 uniforms: mean 0, variance 1 */
    double s = -6.0;
    for (int i = 0; i < 12; ++i) s += uniform();
    return s;
}

static int bucket_of(float x, float lo, float inv_w) {
    volatile float u = x - lo; /* two separately rounded fp32 operations */
    volatile float t = u * inv_w;
    if (!(t > 0.0f)) return 0;
    if (t >= 255.0f) return 255;
    return (int)floorf(t);
}

int main(void) {
    const uint64_t seg[T + 1] = {0, 1000003, 1000003 + 4096, 1000003 + 4096 + 2500001};
    const uint64_t n = seg[T];
    const float lr = 0.7f, beta = 0.9f;
    int bad = 0;

    float* theta = (float*)malloc(n * sizeof(float));
    float* local[W];
    for (int p = 0; p < W; ++p) local[p] = (float*)malloc(n * sizeof(float));
    for (uint64_t i = 0; i < n; ++i) {
        theta[i] = (float)(0.02 * bell());
        for (int p = 0; p < W; ++p) local[p][i] = (float)((double)theta[i] + 1e-3 * bell());
    }

    float *d_theta, *d_local, *d_mom, *d_lut[W], *d_lut2;
    uint8_t *d_codes[W], *d_codes2;
    diloco_qparams *d_qp, *d_qp2;
    void* d_ws;
    const size_t ws_bytes = diloco_workspace_bytes(T);
    HIP_OK(hipMalloc((void**)&d_theta, n * 4));
    HIP_OK(hipMalloc((void**)&d_local, n * 4));
    HIP_OK(hipMalloc((void**)&d_mom, n * 4));
    HIP_OK(hipMalloc((void**)&d_codes2, n));
    HIP_OK(hipMalloc((void**)&d_lut2, T * 256 * 4));
    HIP_OK(hipMalloc((void**)&d_qp, W * T * sizeof(diloco_qparams)));
    HIP_OK(hipMalloc((void**)&d_qp2, T * sizeof(diloco_qparams)));
    HIP_OK(hipMalloc(&d_ws, ws_bytes));
    for (int p = 0; p < W; ++p) {
        HIP_OK(hipMalloc((void**)&d_codes[p], n));
        HIP_OK(hipMalloc((void**)&d_lut[p], T * 256 * 4));
    }
    HIP_OK(hipMemcpy(d_theta, theta, n * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemset(d_mom, 0, n * 4));

    /* stage 1, once per worker (here all on one device, one after the other on the null stream) */
    for (int p = 0; p < W; ++p) {
        HIP_OK(hipMemcpy(d_local, local[p], n * 4, hipMemcpyHostToDevice));
        LIB_OK(diloco_pseudograd_quantize(d_theta, d_local, DILOCO_DTYPE_FP32, n, seg, T, d_codes[p], d_lut[p],
                                          d_qp + p * T, d_ws, ws_bytes, NULL));
        HIP_OK(hipDeviceSynchronize()); /* d_local is overwritten by the next worker's copy */
    }
    /* stage 2 and stage 3 */
    const uint8_t* code_ptrs[W];
    const float* lut_ptrs[W];
    for (int p = 0; p < W; ++p) {
        code_ptrs[p] = d_codes[p];
        lut_ptrs[p] = d_lut[p];
    }
    LIB_OK(int8_reduce_chunk(code_ptrs, lut_ptrs, W, NULL, W, n, seg, T, NULL, d_codes2, d_lut2, d_qp2, d_ws,
                             ws_bytes, NULL));
    LIB_OK(outer_nesterov_step(d_theta, d_mom, NULL, d_codes2, d_lut2, seg, T, n, lr, beta, NULL,
                               DILOCO_DTYPE_FP32, d_ws, ws_bytes, NULL));
    HIP_OK(hipDeviceSynchronize());

    /* results back */
    uint8_t* codes[W];
    float* lut[W];
    diloco_qparams qp[W * T], qp2[T];
    for (int p = 0; p < W; ++p) {
        codes[p] = (uint8_t*)malloc(n);
        lut[p] = (float*)malloc(T * 256 * 4);
        HIP_OK(hipMemcpy(codes[p], d_codes[p], n, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(lut[p], d_lut[p], T * 256 * 4, hipMemcpyDeviceToHost));
    }
    uint8_t* codes2 = (uint8_t*)malloc(n);
    float* lut2 = (float*)malloc(T * 256 * 4);
    float* theta_new = (float*)malloc(n * 4);
    float* mom_new = (float*)malloc(n * 4);
    HIP_OK(hipMemcpy(codes2, d_codes2, n, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(lut2, d_lut2, T * 256 * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(qp, d_qp, sizeof(qp), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(qp2, d_qp2, sizeof(qp2), hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(theta_new, d_theta, n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(mom_new, d_mom, n * 4, hipMemcpyDeviceToHost));

    /* stage 1: statistics and bucket indices */
    for (int p = 0; p < W; ++p)
        for (int s = 0; s < T; ++s) {
            const diloco_qparams* q = &qp[p * T + s];
            const uint64_t a = seg[s], b = seg[s + 1];
            double sum = 0.0, sq = 0.0;
            for (uint64_t i = a; i < b; ++i) sum += (double)(float)(theta[i] - local[p][i]);
            const double mean = sum / (double)(b - a);
            for (uint64_t i = a; i < b; ++i) {
                const double d = (double)(float)(theta[i] - local[p][i]) - mean;
                sq += d * d;
            }
            const double sd = sqrt(sq / (double)(b - a - 1));
            if (q->n != b - a || q->status != 0 || fabs(q->mean - mean) > 1e-9 * sd || fabs(q->std - sd) > 1e-9 * sd) {
                fprintf(stderr, "worker %d tensor %d: statistics differ\n", p, s);
                ++bad;
            }
            if (q->lo != (float)(mean - 6.0 * sd) && fabs((double)q->lo - (mean - 6.0 * sd)) > 1e-6 * sd) ++bad;
            for (uint64_t i = a; i < b; ++i) {
                const float d = theta[i] - local[p][i];
                if (codes[p][i] != bucket_of(d, q->lo, q->inv_w)) {
                    if (bad < 5) fprintf(stderr, "worker %d element %llu: code differs\n", p, (unsigned long long)i);
                    ++bad;
                }
            }
        }
    /* stage 2: fp32 sum of the decoded values in worker order, divided by W, then bucketed with the
       returned range; stage 3: m' = beta m + g, theta' = theta - lr (g + beta m') from m = 0 */
    for (int s = 0; s < T; ++s)
        for (uint64_t i = seg[s]; i < seg[s + 1]; ++i) {
            volatile float acc = 0.0f;
            for (int p = 0; p < W; ++p) acc = acc + lut[p][s * 256 + codes[p][i]];
            volatile float avg = acc / (float)W;
            if (codes2[i] != bucket_of(avg, qp2[s].lo, qp2[s].inv_w)) {
                if (bad < 5) fprintf(stderr, "element %llu: reduced code differs\n", (unsigned long long)i);
                ++bad;
            }
            const float g = lut2[s * 256 + codes2[i]];
            const double m = (double)g, th = (double)theta[i] - (double)lr * ((double)g + (double)beta * m);
            if (fabs((double)mom_new[i] - m) > 1e-6 * fabs(m) || fabs((double)theta_new[i] - th) > 1e-5 * (fabs(th) + fabs(m))) {
                if (bad < 5) fprintf(stderr, "element %llu: outer step differs\n", (unsigned long long)i);
                ++bad;
            }
        }
    printf("example_outer_sync: %llu elements in %d tensors, %d workers: %s\n", (unsigned long long)n, T, W,
           bad ? "MISMATCH" : "OK");
    return bad ? 1 : 0;
}
