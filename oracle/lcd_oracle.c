/*
 * CPU oracle for the LCD smoothed table-lookup linear layer.  TEST INFRASTRUCTURE ONLY:
 * it may be called from tests/, from __graft_entry__.smoke() and from bench.py's
 * cpu_baseline leg, never from the product path.  It shares no code, header, table or
 * constant with the HIP library.
 *
 * What it computes (fp64 throughout, inputs converted exactly):
 *
 *   What[n][k] = C[n][ idx[n][k] ]          -- a clustered weight IS its centroid
 *                                              (paper Sec. 3.2: clustered weights W' and
 *                                              centroids C)
 *   xs[m][k]   = x[m][k] / s[k]             -- inputs are divided by the smoothing factor
 *                                              the weights were multiplied by offline
 *                                              (paper Sec. 3.4, last paragraph)
 *   Y[m][n]    = sum_k xs[m][k] * What[n][k] -- lookup + accumulate equals the product it
 *                                              replaces (paper Sec. 4, Sec. 4.2)
 *
 * The sum runs over k = 0..K-1 in order; there is no blocking, no reordering.  A second
 * entry point evaluates the same result in the "centroid bucket" order of Sec. 4.2
 * (one partial sum of activations per centroid, then one multiply per centroid).
 * A third applies the input-transformation stage of Sec. 4.1 (Eq. 10-11): symmetric
 * uniform quantisation of the smoothed input to b bits.
 *
 * Indices arrive one per byte (never packed): the oracle does not know the GPU layout.
 * Parallelism: OpenMP over output rows n only (each Y[m][n] is still one sequential sum).
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE binary16 bit pattern -> double, written out from the format definition. */
double oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);               /* subnormal: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* What[n][k] = C[n][idx[n][k]].  Returns 0, or 1 if an index is >= 2^bits. */
int oracle_dequant(const uint16_t *codebook, const uint8_t *idx, int N, int K, int bits,
                   double *What)
{
    int ncent = 1 << bits;
    int bad = 0;
    for (int n = 0; n < N; n++) {
        for (int k = 0; k < K; k++) {
            int c = idx[(size_t)n * K + k];
            if (c >= ncent) { bad = 1; c = 0; }
            What[(size_t)n * K + k] = oracle_half_to_double(codebook[(size_t)n * ncent + c]);
        }
    }
    return bad;
}

/* xs[m][k] = x[m][k] / s[k] in fp64. */
void oracle_smooth(const uint16_t *x, const float *s, int M, int K, double *xs)
{
    for (int m = 0; m < M; m++)
        for (int k = 0; k < K; k++)
            xs[(size_t)m * K + k] = oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];
}

/* Y[m][n] = sum_k (x[m][k]/s[k]) * C[n][idx[n][k]], k in order.  Y is [M][N] row-major. */
int oracle_lut_matmul(const uint16_t *codebook, const uint8_t *idx, const uint16_t *x,
                      const float *s, int M, int N, int K, int bits, double *Y)
{
    int ncent = 1 << bits;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int n = 0; n < N; n++) {
        double cent[16];
        for (int c = 0; c < ncent; c++)
            cent[c] = oracle_half_to_double(codebook[(size_t)n * ncent + c]);
        for (int m = 0; m < M; m++) {
            double acc = 0.0;
            for (int k = 0; k < K; k++) {
                int c = idx[(size_t)n * K + k];
                if (c >= ncent) { bad = 1; c = 0; }
                double xs = oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];
                acc += xs * cent[c];
            }
            Y[(size_t)m * N + n] = acc;
        }
    }
    return bad;
}

/* Same result in centroid-bucket order (Sec. 4.2): S[c] = sum_{k: idx[n][k]==c} xs[m][k],
 * then Y[m][n] = sum_c C[n][c] * S[c]. */
int oracle_bucket_matmul(const uint16_t *codebook, const uint8_t *idx, const uint16_t *x,
                         const float *s, int M, int N, int K, int bits, double *Y)
{
    int ncent = 1 << bits;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int n = 0; n < N; n++) {
        for (int m = 0; m < M; m++) {
            double S[16];
            for (int c = 0; c < ncent; c++) S[c] = 0.0;
            for (int k = 0; k < K; k++) {
                int c = idx[(size_t)n * K + k];
                if (c >= ncent) { bad = 1; c = 0; }
                S[c] += oracle_half_to_double(x[(size_t)m * K + k]) / (double)s[k];
            }
            double acc = 0.0;
            for (int c = 0; c < ncent; c++)
                acc += oracle_half_to_double(codebook[(size_t)n * ncent + c]) * S[c];
            Y[(size_t)m * N + n] = acc;
        }
    }
    return bad;
}

/* Input transformation stage (Sec. 4.1, Eq. 10-11) with the two steps fused as the paper
 * describes: q = clip(round_half_even(x / (s_m * s_q)), -2^(b-1), 2^(b-1)-1).
 * The printed range [-2^b, 2^b-1] does not fit b bits; the b-bit symmetric range is used.
 * s_m is per input channel here ([K]); s_q is one scalar. */
void oracle_input_transform(const uint16_t *x, const float *s_m, double s_q, int b,
                            int M, int K, int32_t *q)
{
    double lo = -ldexp(1.0, b - 1), hi = ldexp(1.0, b - 1) - 1.0;
    for (int m = 0; m < M; m++) {
        for (int k = 0; k < K; k++) {
            double v = oracle_half_to_double(x[(size_t)m * K + k]) / ((double)s_m[k] * s_q);
            double r = nearbyint(v); /* default rounding mode: to nearest, ties to even */
            if (r < lo) r = lo;
            if (r > hi) r = hi;
            q[(size_t)m * K + k] = (int32_t)r;
        }
    }
}

/* The same stage in the arithmetic a single-precision kernel uses, step by step:
 * d = s_m * s_q rounded to binary32, v = x / d rounded to binary32, round half to even, clip.
 * Where floating point decides an integer, oracle and kernel must decide in the same precision;
 * this is the kernel's.  (volatile keeps every intermediate in binary32.) */
void oracle_input_transform_f32(const uint16_t *x, const float *s_m, float s_q, int b,
                                int M, int K, int32_t *q)
{
    float lo = -ldexpf(1.0f, b - 1), hi = ldexpf(1.0f, b - 1) - 1.0f;
    for (int m = 0; m < M; m++) {
        for (int k = 0; k < K; k++) {
            volatile float d = s_m[k] * s_q;
            volatile float xf = (float)oracle_half_to_double(x[(size_t)m * K + k]); /* exact */
            volatile float v = xf / d;
            float r = nearbyintf(v);
            if (r < lo) r = lo;
            if (r > hi) r = hi;
            q[(size_t)m * K + k] = (int32_t)r;
        }
    }
}
