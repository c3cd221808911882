/*
 * CPU oracle for the delta-serving linear layer.  TEST INFRASTRUCTURE ONLY: nothing on the product
 * path may call, link or import this file; it shares no code, header, table or helper with the GPU
 * library.  It is deliberately plain and slow.
 *
 * What it computes (paper Section 5.1, Eq. (2), and the SBMM problem statement of Section 5.2):
 * for every request row t with delta index m = Idx[t],
 *
 *     y[t][n] = sum_k x[t][k] * ( W_base[n][k] + Delta_m[n][k] )          (fused result)
 *     y_base  = sum_k x[t][k] * W_base[n][k]                               ("batched fp16 matmul")
 *     y_delta = sum_k x[t][k] * Delta_m[n][k]                              ("quantized sparse matmul")
 *
 * where Delta_m is the dense matrix that the compressed delta stands for.  The compressed delta
 * (Section 4.1, steps 2 and 3) keeps two values out of every four consecutive entries along k
 * together with their 2-bit positions, and stores each kept value as a low-bit code on a group-wise
 * grid: value = (code - zero) * scale.  The decoupling, request reordering, batching and fused
 * dequantisation described in Section 5 are exact re-associations of this definition, so the oracle
 * is the definition itself: dequantise densely, then a dot product per (request, output).
 *
 * Conventions: W and Delta are [N][K] row-major (N = output features, K = input features); the
 * 2:4 groups run along k; x is [T][K]; y is [T][N].  fp16 operands arrive as their 16-bit patterns
 * and are widened exactly; sums run over k in ascending order with one accumulator, in fp32
 * (acc64 == 0) or in fp64 (acc64 != 0, used to show the fp32 oracle's own rounding is negligible).
 * Idx[t] == -1 or outside [0, D) means "base model only".
 *
 * Parity pins (tests/test_oracle_*.py): hand-built code tables with closed-form values, all six
 * position pairs, delta == 0 reproducing the base product bit for bit, linearity, a separately
 * written triple loop on 8x8 tiles, a library sgemm, and numpy's stable argsort for dzo_segment.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* exact IEEE binary16 -> binary32 */
static float half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t e = (h >> 10) & 0x1f;
    uint32_t m = h & 0x3ff;
    uint32_t bits;
    if (e == 0) {
        if (m == 0) {
            bits = sign;
        } else {                       /* subnormal: value = m * 2^-24 */
            float v = (float)m * 5.9604644775390625e-08f;
            memcpy(&bits, &v, 4);
            bits |= sign;
        }
    } else if (e == 31) {
        bits = sign | 0x7f800000u | (m << 13);
    } else {
        bits = sign | ((e + 112) << 23) | (m << 13);
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

int dzo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void dzo_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Check that canonical tables describe a legal compressed delta (Section 4.1 steps 2-3):
 * codes fit in `bits`, the two stored positions of every group of four are distinct and
 * ascending, zero-points are integers on the code range, scales are finite.
 * Returns 0 if legal, otherwise a positive code naming the first kind of violation found.
 */
int dzo_validate(const uint8_t *codes, const uint8_t *idx, const uint16_t *scale,
                 const uint16_t *zero, int N, int K, int bits, int group)
{
    if (N <= 0 || K <= 0) return 1;
    if (bits != 2 && bits != 4) return 2;
    if (group <= 0 || group % 4 != 0 || K % group != 0) return 3;
    const int qmax = (1 << bits) - 1;
    const size_t half = (size_t)K / 2;
    int bad = 0;
    for (int n = 0; n < N && !bad; ++n) {
        for (size_t j = 0; j < half; ++j)
            if (codes[n * half + j] > qmax) { bad = 4; break; }
        for (size_t g = 0; g < half / 2 && !bad; ++g) {
            uint8_t a = idx[n * half + 2 * g], b = idx[n * half + 2 * g + 1];
            if (a > 3 || b > 3 || !(a < b)) bad = 5;
        }
        for (int g = 0; g < K / group && !bad; ++g) {
            float z = half_to_float(zero[(size_t)n * (K / group) + g]);
            float s = half_to_float(scale[(size_t)n * (K / group) + g]);
            if (!(z >= 0.0f && z <= (float)qmax) || z != floorf(z)) bad = 6;
            if (!isfinite(s)) bad = 7;
        }
    }
    return bad;
}

/*
 * Dense fp32 matrix that the tables stand for: the kept value j (0 or 1) of the g-th group of
 * four in row n goes to column 4g + idx, everything else is zero; its value is
 * (code - zero) * scale with the zero/scale of the quantisation group that column 4g lies in.
 * |code - zero| < 16 and an fp16 scale has an 11-bit significand, so the fp32 product is exact.
 */
void dzo_dequant(const uint8_t *codes, const uint8_t *idx, const uint16_t *scale,
                 const uint16_t *zero, int N, int K, int bits, int group, float *dense)
{
    (void)bits;
    const size_t half = (size_t)K / 2;
    const int ngroups = K / group;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        float *row = dense + (size_t)n * K;
        for (int k = 0; k < K; ++k) row[k] = 0.0f;
        for (int g = 0; g < K / 4; ++g) {
            const int qg = (4 * g) / group;
            const float s = half_to_float(scale[(size_t)n * ngroups + qg]);
            const float z = half_to_float(zero[(size_t)n * ngroups + qg]);
            for (int j = 0; j < 2; ++j) {
                const size_t e = n * half + 2 * (size_t)g + j;
                row[4 * g + idx[e]] = ((float)codes[e] - z) * s;
            }
        }
    }
}

/*
 * y[t][n] = sum_k x[t][k] * (W[n][k] + Delta_{Idx[t]}[n][k]).
 *   W      : fp16 [N][K], or NULL for "no base term" (gives y_delta)
 *   deltas : D pointers to dense fp32 [N][K] matrices from dzo_dequant, or NULL / D == 0 for
 *            "no delta term" (gives y_base)
 *   idx    : int32 [T]; a value outside [0, D) selects no delta
 *   acc64  : 0 -> fp32 operands' sum W+Delta in fp32 and fp32 accumulator;
 *            1 -> the same in fp64
 */
void dzo_linear(const uint16_t *x, const uint16_t *W, const float *const *deltas, int D,
                const int32_t *idx, int T, int N, int K, int acc64, float *y)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int t = 0; t < T; ++t) {
            const int m = idx ? idx[t] : -1;
            const float *drow = (deltas && m >= 0 && m < D) ? deltas[m] + (size_t)n * K : NULL;
            const uint16_t *wrow = W ? W + (size_t)n * K : NULL;
            const uint16_t *xrow = x + (size_t)t * K;
            if (acc64) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k) {
                    double w = wrow ? (double)half_to_float(wrow[k]) : 0.0;
                    if (drow) w += (double)drow[k];
                    acc += (double)half_to_float(xrow[k]) * w;
                }
                y[(size_t)t * N + n] = (float)acc;
            } else {
                float acc = 0.0f;
                for (int k = 0; k < K; ++k) {
                    float w = wrow ? half_to_float(wrow[k]) : 0.0f;
                    if (drow) w += drow[k];
                    acc += half_to_float(xrow[k]) * w;
                }
                y[(size_t)t * N + n] = acc;
            }
        }
    }
}

/*
 * Request reordering (Section 5.2, first optimisation): group the requests of one delta together.
 * Stable counting sort of Idx: counts[m] = number of requests of delta m, offsets = exclusive
 * prefix sum (offsets[D] = number of requests that have a delta), perm lists request indices
 * delta by delta, each delta's requests in their original order; requests whose index is outside
 * [0, D) (base model only) follow at the end, also in original order.
 */
void dzo_segment(const int32_t *idx, int T, int D, int32_t *counts, int32_t *offsets,
                 int32_t *perm)
{
    for (int m = 0; m < D; ++m) counts[m] = 0;
    for (int t = 0; t < T; ++t)
        if (idx[t] >= 0 && idx[t] < D) counts[idx[t]]++;
    offsets[0] = 0;
    for (int m = 0; m < D; ++m) offsets[m + 1] = offsets[m] + counts[m];
    int32_t tail = offsets[D];
    for (int m = 0; m < D; ++m) {
        int32_t p = offsets[m];
        for (int t = 0; t < T; ++t)
            if (idx[t] == m) perm[p++] = t;
    }
    for (int t = 0; t < T; ++t)
        if (!(idx[t] >= 0 && idx[t] < D)) perm[tail++] = t;
}
