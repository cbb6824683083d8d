/*
 * Plain C oracle for the Matryoshka-sliced quantized linear layer.
 *
 * TEST INFRASTRUCTURE ONLY: used by tests/ (cross-checked against the numpy
 * oracle and the same pins) and by the cpu_baseline leg of bench.py.  It shares
 * no code with the HIP path and the product never links it.
 *
 * The three steps, in the paper's order, one weight at a time:
 *   Eq. 1 (Section 2):       S = clamp(round(q / 2^(c-r)), 0, 2^r-1) * 2^(c-r)
 *                            (round half up; r == c is the identity)
 *   Section 3.2, item 1:     w = scale * (S - zero), scale/zero of the master
 *                            width c, groups contiguous along the input dim
 *   Section 4:               y = x W^T, fp16 inputs, wide accumulator (double)
 *
 * fp16 values travel as their 16 raw bits (uint16_t).
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)mant, -24);               /* subnormal or zero */
    else if (expo == 31)
        v = mant ? NAN : INFINITY;
    else
        v = ldexp((double)(mant + 1024), expo - 25); /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* Eq. 1 for one code.  Returns the c-bit grid value S. */
static int slice_one(int q, int c, int r)
{
    int step = 1 << (c - r);
    int t = (2 * q + step) / (2 * step);            /* round half up, q >= 0 */
    int tmax = (1 << r) - 1;
    if (t < 0) t = 0;
    if (t > tmax) t = tmax;
    return t * step;
}

int mqo_slice(const uint8_t *q, int64_t n, int c, int r, uint8_t *S)
{
    if (!q || !S || c < 1 || c > 8 || r < 1 || r > c) return -1;
    for (int64_t i = 0; i < n; ++i) S[i] = (uint8_t)slice_one(q[i], c, r);
    return 0;
}

/* y[m*N + n] = sum_k x[m,k] * scale[n,k/group] * (S(parent[n,k]) - zero[n,k/group]).
 * Returns the number of threads used, or -1 on bad arguments. */
int mqo_linear(const uint16_t *x, int64_t M, const uint8_t *parent,
               const uint16_t *scales, const uint16_t *zeros,
               int64_t N, int64_t K, int c, int r, int group, double *y)
{
    if (!x || !parent || !scales || !zeros || !y) return -1;
    if (c < 1 || c > 8 || r < 1 || r > c || group <= 0 || K % group) return -1;
    int64_t G = K / group;
    int used = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#pragma omp parallel for schedule(static)
#endif
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                int64_t g = k / group;
                double s = half_bits_to_double(scales[n * G + g]);
                double z = half_bits_to_double(zeros[n * G + g]);
                double S = (double)slice_one(parent[n * K + k], c, r);
                double w = s * (S - z);
                acc += half_bits_to_double(x[m * K + k]) * w;
            }
            y[m * N + n] = acc;
        }
    }
    return used;
}
