/*
 * CPU oracle for the weight-only-quantized fully-connected layer.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or
 * import this file; it exists so that the GPU kernels can be checked against a
 * slow, plain, obviously correct implementation.  It shares no code with the
 * GPU library.
 *
 * What it follows:
 *   - the statement of the quantized linear layer and its two stages
 *     (section 3.7, "Stage-Aware Optimizations for LLM Inference"): prefill
 *     quantizes the float activations to 8-bit integers with their quantization
 *     parameters, multiplies them with pre-quantized weights using integer
 *     arithmetic and dequantizes the output; decode is a fully connected
 *     kernel over the same weights;
 *   - the weight formats of section 4.2: per-channel int8 ("q8") and int4
 *     ("8/4/4"), and sub-channel (group) quantization named in the conclusion
 *     as the next scheme, instantiated here as groups of 32 along K;
 *   - FP16 activations (section 4.2).
 *
 * Weight-only path: the result has a plain definition, y = x . dequant(W)^T,
 * so the oracle is that definition written out: dequantize every weight into a
 * double matrix, then a triple loop in fp64 with k ascending.
 *
 * Integer path: an encoding (activation quantization, fp32 arithmetic in the
 * order stated below) followed by an exact integer contraction and a rescale;
 * the oracle takes those steps one by one.
 *
 * All functions are pinned by tests/test_oracle_pins.py (exact-rational brute
 * force, closed forms, library special cases, invariants); none is "parity
 * unpinned".
 *
 * Build: gcc -O2 -fno-fast-math -ffp-contract=off -fopenmp -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads the loops below will use (reported beside timings). */
int qfc_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* IEEE binary16 bit pattern -> double, exactly (every binary16 value is a
 * double).  Written from the format definition: 1 sign, 5 exponent (bias 15),
 * 10 fraction bits; exponent 0 is subnormal, 31 is inf/nan. */
double qfc_oracle_f16_to_f64(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

/* Dequantize per-output-channel int8 (or int4-in-int8) weights:
 * What[n,k] = s[n] * Wq[n,k], scale fp32 per output channel (section 4.2,
 * "per-channel"; the channel is the output channel O of the OHWI layout of
 * section 3.1, the only axis that factors out of the sum over K). */
void qfc_oracle_dequant_per_channel(const int8_t *wq, const float *s, int64_t N,
                                    int64_t K, double *what) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            what[n * K + k] = (double)s[n] * (double)wq[n * K + k];
}

/* Dequantize group quantized weights: one binary16 scale per `group`
 * consecutive k of one output row, scales laid out [N, K/group]
 * (sub-channel quantization; group = 32 in every workload here). */
void qfc_oracle_dequant_group(const int8_t *wq, const uint16_t *s_f16, int64_t N,
                              int64_t K, int64_t group, double *what) {
    int64_t G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            what[n * K + k] = qfc_oracle_f16_to_f64(s_f16[n * G + k / group]) *
                              (double)wq[n * K + k];
}

/* y[m,n] = sum_k x[m,k] * What[n,k], fp64, k ascending; x is binary16. The
 * result is kept in fp64 (never rounded to binary16). */
void qfc_oracle_fc_f64(const uint16_t *x_f16, const double *what, int64_t M,
                       int64_t N, int64_t K, double *y) {
    double *xd = (double *)malloc(sizeof(double) * (size_t)(M * K));
    for (int64_t i = 0; i < M * K; ++i) xd[i] = qfc_oracle_f16_to_f64(x_f16[i]);
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += xd[m * K + k] * what[n * K + k];
            y[m * N + n] = acc;
        }
    free(xd);
}

/* Dynamic per-token symmetric int8 quantization of the activations (the
 * "quantization kernel" of section 3.7; granularity, rounding and the scale
 * formula are this build's reading, stated in the design notes):
 *   a     = max_k |x[m,k]|                      (exact)
 *   sx[m] = a / 127            one fp32 division
 *   inv   = 127 / a            one fp32 division
 *   xq    = clamp(rint(x*inv)) one fp32 multiply, then round-half-to-even
 * An all-zero row gives sx = 0 and xq = 0.  Everything is fp32 on purpose:
 * the GPU has to reproduce these bits. */
void qfc_oracle_quantize_activations(const uint16_t *x_f16, int64_t M, int64_t K,
                                     int8_t *xq, float *sx) {
    for (int64_t m = 0; m < M; ++m) {
        float a = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float v = fabsf((float)qfc_oracle_f16_to_f64(x_f16[m * K + k]));
            if (v > a) a = v;
        }
        float scale = 0.0f, inv = 0.0f;
        if (a != 0.0f) {
            scale = a / 127.0f;
            inv = 127.0f / a;
        }
        sx[m] = scale;
        for (int64_t k = 0; k < K; ++k) {
            float v = (float)qfc_oracle_f16_to_f64(x_f16[m * K + k]);
            volatile float p = v * inv; /* one rounding, no fused contraction */
            float r = rintf(p);
            if (r > 127.0f) r = 127.0f;
            if (r < -127.0f) r = -127.0f;
            xq[m * K + k] = (int8_t)r;
        }
    }
}

/* acc[m,n] = sum_k xq[m,k] * Wq[n,k], exact (int64). */
void qfc_oracle_int_contract(const int8_t *xq, const int8_t *wq, int64_t M,
                             int64_t N, int64_t K, int64_t *acc) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            int64_t a = 0;
            for (int64_t k = 0; k < K; ++k)
                a += (int64_t)xq[m * K + k] * (int64_t)wq[n * K + k];
            acc[m * N + n] = a;
        }
}

/* Output dequantization: y[m,n] = acc[m,n] * sx[m] * sw[n] in fp64. */
void qfc_oracle_rescale(const int64_t *acc, const float *sx, const float *sw,
                        int64_t M, int64_t N, double *y) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            y[m * N + n] = (double)acc[m * N + n] * (double)sx[m] * (double)sw[n];
}
