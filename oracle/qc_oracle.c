/*
 * CPU oracle for the quantized-linear hot path of QuantCache (arxiv 2503.06545).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and the
 * product never calls it: only the tests, the smoke check and the benchmark's
 * CPU-baseline leg load it.
 *
 * What it follows in the paper:
 *   - uniform quantizer, Section 3.1 "Model Quantization", Eq. (3) and Eq. (4)
 *     (third and fourth displayed equations), taken in its symmetric signed
 *     form: range [-a, +a], 2^b - 1 levels, zero point at mid range, so the
 *     stored code is rne(x / s) with s = a / (2^(b-1) - 1); and, for
 *     activations, also as printed (orc_quant_rows_asym): unsigned codes with
 *     a zero point per token, s = (max - min) / (2^b - 1);
 *   - Section 4.1 "Quantization Scheme": one scale per output channel of a
 *     weight, activation scales computed online (here: one per token row);
 *   - Section 3.2 AIGQ (1): the weight bit-width is chosen per layer, so the
 *     quantizer takes qmax (127 for 8 bit, 7 for 4 bit) as an argument;
 *   - Section 4.1 "Hardware Implementation": the linear layer runs as a
 *     low-bit integer GEMM with the (de)quantization fused around it;
 *   - Section 3.2 HLC, Eq. (5): the L1 norm of the change of a latent between
 *     the current and the cached step; its second factor, the norm of the
 *     inter-frame gradient of the feature map, is named there and not defined.
 *     orc_frame_gradient takes one reading of it (forward difference along the
 *     frame axis, Euclidean norm).  The arithmetic of that reading is pinned by
 *     the tests; that it is the authors' definition cannot be checked from the
 *     paper: parity unpinned for this function in that sense;
 *   - Section 3.3 SRAP, Eq. (9) (cosine similarity of consecutive layers) and
 *     Eq. (11) (cumulative L1 variation over the previous steps);
 *   - Section 3.2 AIGQ (1) and Section 4.1 "Hardware Implementation": a rotation
 *     applied together with the quantization.  The matrix is not given; the
 *     reading here is a block Walsh-Hadamard transform (orc_rotate_rows_f32).
 *     Its arithmetic is pinned (the explicit matrix, H H^T = block * I, the
 *     unchanged product X W^T); which rotation the authors use is not:
 *     parity unpinned in that sense.
 *
 * Arithmetic contract.  The steps marked [bit] are single IEEE-754 binary32
 * operations, round to nearest even, written one per statement so that no
 * reassociation or contraction can apply (build with -ffp-contract=off and
 * never with -ffast-math).  Everything else is binary64.
 *
 * All loops are the naive ones.  The only parallelism is an OpenMP
 * "parallel for" over independent rows so the same code can be timed on all
 * host cores.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* smallest absmax used for a scale: an exact power of two, keeps s normal */
#define ORC_ABSMAX_FLOOR 0x1p-64f

enum { ORC_EPI_NONE = 0, ORC_EPI_GELU_TANH = 1, ORC_EPI_GELU_ERF = 2 };

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* bf16 -> binary32 is exact: the 16 bits are the top half of the float. */
static float bf16_bits_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* binary32 -> bf16, round to nearest even on the 16 dropped bits. */
static uint16_t f32_to_bf16_bits(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN */
    uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
    return (uint16_t)upper;
}

/*
 * One row of the symmetric quantizer (Eq. (3), Eq. (4), symmetric reading):
 *   a = max_k |x_k|                               [bit] (exact in any order)
 *   s = max(a, 2^-64) / qmax                      [bit]
 *   q_k = clamp(rne(x_k / s), -qmax, +qmax)       [bit]
 */
static void quant_row(const float *x, int64_t K, int qmax, int8_t *q, float *s_out) {
    float a = 0.0f;
    for (int64_t k = 0; k < K; ++k) {
        float v = fabsf(x[k]);
        if (v > a) a = v;
    }
    float floored = a > ORC_ABSMAX_FLOOR ? a : ORC_ABSMAX_FLOOR;
    float s = floored / (float)qmax;
    for (int64_t k = 0; k < K; ++k) {
        float t = x[k] / s;
        float r = rintf(t); /* default rounding mode: ties to even */
        if (r > (float)qmax) r = (float)qmax;
        if (r < -(float)qmax) r = -(float)qmax;
        q[k] = (int8_t)r;
    }
    *s_out = s;
}

/* Rows of a float matrix [R, K] -> codes [R, K] and scales [R]. */
void orc_quant_rows_f32(const float *X, int64_t R, int64_t K, int qmax, int8_t *q, float *s) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r) quant_row(X + r * K, K, qmax, q + r * K, s + r);
}

/* Same for a bf16 matrix given as raw 16-bit patterns. */
void orc_quant_rows_bf16(const uint16_t *X, int64_t R, int64_t K, int qmax, int8_t *q, float *s) {
#pragma omp parallel
    {
        float *tmp = (float *)malloc((size_t)(K > 0 ? K : 1) * sizeof(float));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < R; ++r) {
            for (int64_t k = 0; k < K; ++k) tmp[k] = bf16_bits_to_f32(X[r * K + k]);
            quant_row(tmp, K, qmax, q + r * K, s + r);
        }
        free(tmp);
    }
}

/*
 * Canonical int4 container: byte j of a row holds code 2j in bits 0..3 and
 * code 2j+1 in bits 4..7, each as a 4-bit two's complement number.
 */
void orc_pack_int4(const int8_t *codes, int64_t N, int64_t K, uint8_t *packed) {
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t lo = (uint8_t)codes[n * K + 2 * j] & 0x0fu;
            uint8_t hi = (uint8_t)codes[n * K + 2 * j + 1] & 0x0fu;
            packed[n * (K / 2) + j] = (uint8_t)(lo | (hi << 4));
        }
}

void orc_unpack_int4(const uint8_t *packed, int64_t N, int64_t K, int8_t *codes) {
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < K / 2; ++j) {
            uint8_t b = packed[n * (K / 2) + j];
            int lo = b & 0x0f, hi = (b >> 4) & 0x0f;
            codes[n * K + 2 * j] = (int8_t)(lo >= 8 ? lo - 16 : lo);
            codes[n * K + 2 * j + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
        }
}

/* acc[m, n] = sum_k qx[m, k] * qw[n, k], int32, plain triple loop. */
void orc_gemm_i32(const int8_t *qx, const int8_t *qw, int64_t M, int64_t N, int64_t K,
                  int32_t *acc) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t a = 0;
            for (int64_t k = 0; k < K; ++k) a += (int32_t)qx[m * K + k] * (int32_t)qw[n * K + k];
            acc[m * N + n] = a;
        }
}

/* The same sum in int64, to show once that int32 never wraps at these sizes. */
void orc_gemm_i64(const int8_t *qx, const int8_t *qw, int64_t M, int64_t N, int64_t K,
                  int64_t *acc) {
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t a = 0;
            for (int64_t k = 0; k < K; ++k) a += (int64_t)qx[m * K + k] * (int64_t)qw[n * K + k];
            acc[m * N + n] = a;
        }
}

static double gelu_tanh(double y) {
    const double c = 0.79788456080286535588; /* sqrt(2/pi) */
    return 0.5 * y * (1.0 + tanh(c * (y + 0.044715 * y * y * y)));
}

static double gelu_erf(double y) { return 0.5 * y * (1.0 + erf(y * 0.70710678118654752440)); }

/*
 * Dequantize + bias + optional GELU, in binary64:
 *   y[m, n] = acc[m, n] * sx[m] * sw[n] + bias[n]
 * bias may be NULL.
 */
void orc_epilogue_f64(const int32_t *acc, const float *sx, const float *sw, const float *bias,
                      int epi, int64_t M, int64_t N, double *y) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double v = (double)acc[m * N + n] * (double)sx[m] * (double)sw[n];
            if (bias) v += (double)bias[n];
            if (epi == ORC_EPI_GELU_TANH) v = gelu_tanh(v);
            else if (epi == ORC_EPI_GELU_ERF) v = gelu_erf(v);
            y[m * N + n] = v;
        }
}

/* One rounding to the output type. */
void orc_round_to_f32(const double *y, int64_t count, float *out) {
    for (int64_t i = 0; i < count; ++i) out[i] = (float)y[i];
}

void orc_round_to_bf16(const double *y, int64_t count, uint16_t *out) {
    for (int64_t i = 0; i < count; ++i) out[i] = f32_to_bf16_bits((float)y[i]);
}

/*
 * The whole quantized linear on already quantized weights, as the GPU call
 * sees it: quantize the rows of X (act_qmax = 127, or 31 / 7 for the 6- and 4-bit
 * activations of Section 3.2 AIGQ (2), Eq. (8)), integer GEMM, epilogue.  x_is_bf16
 * selects how X is read.  Outputs: codes qx [M, K], scales sx [M], accumulators
 * acc [M, N] and y [M, N] in binary64 (the caller rounds once).
 */
void orc_qlinear(const void *X, int x_is_bf16, int64_t M, int64_t K, int act_qmax,
                 const int8_t *qw, const float *sw, int64_t N, const float *bias, int epi,
                 int8_t *qx, float *sx, int32_t *acc, double *y) {
    if (x_is_bf16)
        orc_quant_rows_bf16((const uint16_t *)X, M, K, act_qmax, qx, sx);
    else
        orc_quant_rows_f32((const float *)X, M, K, act_qmax, qx, sx);
    orc_gemm_i32(qx, qw, M, N, K, acc);
    orc_epilogue_f64(acc, sx, sw, bias, epi, M, N, y);
}

/*
 * Latent change, numerator of Eq. (5) and the norm it is set against:
 *   num = sum_i |cur_i - prev_i|,  den = sum_i |prev_i|,  rel = num / den
 * Sequential binary64 sums.  den == 0: rel = +inf if num > 0, else 0.
 */
void orc_latent_delta(const float *cur, const float *prev, int64_t n, double out[3]) {
    double num = 0.0, den = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        num += fabs((double)cur[i] - (double)prev[i]);
        den += fabs((double)prev[i]);
    }
    out[0] = num;
    out[1] = den;
    if (den > 0.0) out[2] = num / den;
    else out[2] = num > 0.0 ? INFINITY : 0.0;
}

/*
 * Cosine similarity of the features of two consecutive layers (Section 3.3 SRAP, Eq. (9)):
 *   S = <a, b> / (||a|| ||b||), sequential binary64 sums; S = 0 if either norm is 0.
 * out: { <a,b>, <a,a>, <b,b>, S }.  a_is_bf16 selects how both inputs are read.
 */
void orc_layer_similarity(const void *a, const void *b, int is_bf16, int64_t n, double out[4]) {
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double x, y;
        if (is_bf16) {
            x = (double)bf16_bits_to_f32(((const uint16_t *)a)[i]);
            y = (double)bf16_bits_to_f32(((const uint16_t *)b)[i]);
        } else {
            x = (double)((const float *)a)[i];
            y = (double)((const float *)b)[i];
        }
        ab += x * y;
        aa += x * x;
        bb += y * y;
    }
    out[0] = ab;
    out[1] = aa;
    out[2] = bb;
    double denom = sqrt(aa) * sqrt(bb);
    out[3] = denom > 0.0 ? ab / denom : 0.0;
}

/*
 * Inter-frame gradient of a feature map (Section 3.2 HLC, the second factor of Eq. (5)).
 * The paper names the factor and does not define it; the reading taken here: m is laid out
 * [frames, inner], the gradient is the forward difference along the frame axis,
 * g[f, j] = m[f+1, j] - m[f, j] for f < frames-1, and the norm is the Euclidean norm over
 * all of g.  out: { sum g^2, sqrt of it }.  One frame gives 0.
 */
void orc_frame_gradient(const void *m, int is_bf16, int64_t frames, int64_t inner, double out[2]) {
    double ss = 0.0;
    for (int64_t f = 0; f + 1 < frames; ++f)
        for (int64_t j = 0; j < inner; ++j) {
            double lo, hi;
            if (is_bf16) {
                lo = (double)bf16_bits_to_f32(((const uint16_t *)m)[f * inner + j]);
                hi = (double)bf16_bits_to_f32(((const uint16_t *)m)[(f + 1) * inner + j]);
            } else {
                lo = (double)((const float *)m)[f * inner + j];
                hi = (double)((const float *)m)[(f + 1) * inner + j];
            }
            ss += (hi - lo) * (hi - lo);
        }
    out[0] = ss;
    out[1] = sqrt(ss);
}

/*
 * Cumulative feature variation over the previous steps (Section 3.3 SRAP, Eq. (11)):
 *   V = sum_i || p_t - p_{t-i} ||_1.   prevs holds the `count` earlier tensors back to back,
 * [count, n]; the i = 0 term of the printed sum is identically zero and is not stored.
 * out: the `count` L1 distances, then V.
 */
void orc_cumulative_variation(const float *cur, const float *prevs, int count, int64_t n,
                              double *out) {
    double total = 0.0;
    for (int c = 0; c < count; ++c) {
        double d = 0.0;
        for (int64_t i = 0; i < n; ++i)
            d += fabs((double)cur[i] - (double)prevs[(int64_t)c * n + i]);
        out[c] = d;
        total += d;
    }
    out[count] = total;
}

/*
 * Rotation before quantization (Section 3.2 AIGQ (1): a lightweight rotation evens out the
 * channels; Section 4.1 "Hardware Implementation": it is fused with the quantization).  The
 * paper does not give the matrix.  Reading taken here: a block-diagonal Walsh-Hadamard
 * matrix over the reduction axis, blocks of `block` consecutive columns (a power of two that
 * divides K), Sylvester (natural) order, entries +1 / -1.  Since H H^T = block * I, rotating
 * the activations by H and the weights by H / block leaves X W^T unchanged.
 *
 * Arithmetic [bit]: the transform is evaluated as the fast butterfly network in binary32,
 * stages in ascending stride h = 1, 2, 4, ..., block / 2; a stage replaces every pair
 * (x[j], x[j + h]) with bit h of j clear by (x[j] + x[j + h], x[j] - x[j + h]), one rounding
 * each.  The result is multiplied by post_scale (1, or the exact power of two 1 / block).
 * The quantizer then decides codes on these binary32 values, so this order is part of the
 * bit-exact contract with the GPU path.
 */
void orc_rotate_rows_f32(const float *X, int64_t R, int64_t K, int block, float post_scale,
                         float *out) {
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < R; ++r) {
        const float *x = X + r * K;
        float *y = out + r * K;
        for (int64_t k = 0; k < K; ++k) y[k] = x[k];
        for (int64_t b0 = 0; b0 + block <= K; b0 += block) {
            float *v = y + b0;
            for (int h = 1; h < block; h <<= 1)
                for (int j = 0; j < block; ++j)
                    if ((j & h) == 0) {
                        volatile float sum = v[j] + v[j + h];
                        volatile float dif = v[j] - v[j + h];
                        v[j] = sum;
                        v[j + h] = dif;
                    }
            for (int j = 0; j < block; ++j) {
                volatile float scaled = v[j] * post_scale;
                v[j] = scaled;
            }
        }
    }
}

/*
 * The quantizer of Section 3.1 in its printed, asymmetric form, one row (a token):
 *   Eq. (4):  s = (max(x) - min(x)) / (2^b - 1)
 *   Eq. (3):  x_int = clamp(rne(x / s) + z, 0, 2^b - 1)
 * The paper does not print z; the usual choice that sends min(x) to code 0 is taken:
 *   z = -rne(min(x) / s),   dequantized value  s * (x_int - z).
 * levels = 2^b - 1 (255, 63 or 15).  Steps, each one binary32 operation [bit]:
 *   range = hi - lo;  s = max(range, 2^-64) / levels;  z = -rne(lo / s);
 *   x_int = clamp(rne(x / s) + z, 0, levels)   (the sum of two integer-valued floats)
 * z is kept as an integer-valued float: for a row far from zero with a narrow range it
 * exceeds every integer type that would be natural here.
 */
static void quant_row_asym(const float *x, int64_t K, int levels, uint8_t *q, float *s_out,
                           float *z_out) {
    float lo = x[0], hi = x[0];
    for (int64_t k = 1; k < K; ++k) {
        if (x[k] < lo) lo = x[k];
        if (x[k] > hi) hi = x[k];
    }
    float range = hi - lo;
    float floored = range > ORC_ABSMAX_FLOOR ? range : ORC_ABSMAX_FLOOR;
    float s = floored / (float)levels;
    float lo_over_s = lo / s;
    float z = -rintf(lo_over_s);
    for (int64_t k = 0; k < K; ++k) {
        float t = x[k] / s;
        float v = rintf(t) + z;
        if (v < 0.0f) v = 0.0f;
        if (v > (float)levels) v = (float)levels;
        q[k] = (uint8_t)v;
    }
    *s_out = s;
    *z_out = z;
}

void orc_quant_rows_asym(const void *X, int x_is_bf16, int64_t R, int64_t K, int levels,
                         uint8_t *q, float *s, float *z) {
#pragma omp parallel
    {
        float *tmp = (float *)malloc((size_t)(K > 0 ? K : 1) * sizeof(float));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < R; ++r) {
            for (int64_t k = 0; k < K; ++k)
                tmp[k] = x_is_bf16 ? bf16_bits_to_f32(((const uint16_t *)X)[r * K + k])
                                   : ((const float *)X)[r * K + k];
            quant_row_asym(tmp, K, levels, q + r * K, s + r, z + r);
        }
        free(tmp);
    }
}

/*
 * The linear layer on asymmetric activation codes and symmetric weight codes, written as the
 * product of the dequantized operands:
 *   y[m, n] = act( sx[m] * sw[n] * sum_k (qx[m, k] - z[m]) * qw[n, k]  + bias[n] )
 * The sum is exact in binary64 (integer-valued terms far below 2^53 for any sane row).
 */
void orc_qlinear_asym(const void *X, int x_is_bf16, int64_t M, int64_t K, int levels,
                      const int8_t *qw, const float *sw, int64_t N, const float *bias, int epi,
                      uint8_t *qx, float *sx, float *zx, double *y) {
    orc_quant_rows_asym(X, x_is_bf16, M, K, levels, qx, sx, zx);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double a = 0.0;
            for (int64_t k = 0; k < K; ++k)
                a += ((double)qx[m * K + k] - (double)zx[m]) * (double)qw[n * K + k];
            double v = a * (double)sx[m] * (double)sw[n] + (bias ? (double)bias[n] : 0.0);
            if (epi == ORC_EPI_GELU_TANH) v = gelu_tanh(v);
            else if (epi == ORC_EPI_GELU_ERF) v = gelu_erf(v);
            y[m * N + n] = v;
        }
}
