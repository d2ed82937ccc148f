/*
 * CPU oracle for BRACE robust chunk aggregation, plain C -- TEST INFRASTRUCTURE ONLY.
 *
 * The direct definition (Sec. 3 Phase III, Eq. (1); App. A restatement
 * 2*I(sum > lambda) - 1) written out coordinate by coordinate, for inputs too
 * large for the numpy oracle.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may load this library; the product path never does, and
 * this file shares nothing with it.
 *
 * Readings where the paper is silent (same as the numpy oracle):
 *   sign(+0) = sign(-0) = sign(NaN) = zero_sign (0 unless asked otherwise);
 *   packed output is LSB-first, bit set <=> +1.            [parity unpinned]
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC -o liboracle_brace.so brace_oracle.c
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads a parallel region would use when asked for `threads`
 * (<= 0: the runtime default). */
int oracle_threads(int threads)
{
#ifdef _OPENMP
    if (threads > 0)
        return threads;
    return omp_get_max_threads();
#else
    (void)threads;
    return 1;
#endif
}

/* Phase I for one value. */
static int sign_of(float x, int zero_sign)
{
    if (x > 0.0f)
        return 1;
    if (x < 0.0f)
        return -1;
    return zero_sign;
}

/*
 * updates: n rows of d floats, row i starting at updates + i*ld (ld >= d).
 * For every coordinate k: S = sum_i sign(updates[i][k]); out[k] = S > lambda ? +1 : -1.
 * out   : d floats, or NULL.
 * sums  : d int32 sign-sums, or NULL.
 * bits  : ceil(d/8) bytes, or NULL.
 * threads <= 0: OpenMP default.  Returns 0, or -1 on invalid arguments.
 */
int oracle_brace_direct(const float *updates, int64_t n, int64_t d, int64_t ld,
                        double lambda, int zero_sign,
                        float *out, int32_t *sums, uint8_t *bits, int threads)
{
    if (!updates || n < 1 || d < 0 || ld < d || !isfinite(lambda) ||
        zero_sign < -1 || zero_sign > 1)
        return -1;
#ifdef _OPENMP
    int nt = oracle_threads(threads);
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (int64_t k = 0; k < d; ++k) {
        int64_t s = 0;
        for (int64_t i = 0; i < n; ++i)
            s += sign_of(updates[i * ld + k], zero_sign);
        if (sums)
            sums[k] = (int32_t)s;
        if (out)
            out[k] = ((double)s > lambda) ? 1.0f : -1.0f;
    }
    if (bits) {
        /* serial: neighbouring coordinates share a byte */
        int64_t nbytes = (d + 7) / 8;
        for (int64_t b = 0; b < nbytes; ++b)
            bits[b] = 0;
        for (int64_t k = 0; k < d; ++k) {
            int64_t s = 0;
            for (int64_t i = 0; i < n; ++i)
                s += sign_of(updates[i * ld + k], zero_sign);
            if ((double)s > lambda)
                bits[k >> 3] |= (uint8_t)(1u << (k & 7));
        }
    }
    return 0;
}

/*
 * Plain RAR result (Sec. 2.2): sum_i updates[i][k], accumulated in double in
 * client order 0..n-1.  scale multiplies the final sum (1 for the sum, 1/n
 * for the Mean rule of Sec. 2.1).
 */
int oracle_rar_sum(const float *updates, int64_t n, int64_t d, int64_t ld,
                   double scale, double *out, int threads)
{
    if (!updates || !out || n < 1 || d < 0 || ld < d)
        return -1;
#ifdef _OPENMP
    int nt = oracle_threads(threads);
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (int64_t k = 0; k < d; ++k) {
        double s = 0.0;
        for (int64_t i = 0; i < n; ++i)
            s += (double)updates[i * ld + k];
        out[k] = s * scale;
    }
    return 0;
}

/*
 * Plain RAR as a ring of fp32 clients delivers it (Sec. 2.2, Share-Reduce): chunk c starts
 * as client c's sub-vector and every following client on the ring adds its own, so
 * coordinate k of chunk c is ((g_c + g_{c+1}) + ...) + g_{c-1} (indices mod n), each +
 * rounded to float.  Chunks: the first d mod n hold one coordinate more.  With mean != 0
 * the sum is divided by n once, in float (Mean rule of Sec. 2.1).
 *
 * `updates` holds the columns [k0, k0 + width) of the n x d_total matrix (row i at
 * updates + i*ld), so that a large matrix can be checked in column tiles; the chunk of a
 * column is that of its position k0 + j in the full vector.  out: width floats.
 */
int oracle_rar_sum_ring_f32(const float *updates, int64_t n, int64_t width, int64_t ld,
                            int64_t d_total, int64_t k0, int mean, float *out, int threads)
{
    if (!updates || !out || n < 1 || width < 0 || ld < width || k0 < 0 || d_total < k0 + width)
        return -1;
    const int64_t q = d_total / n, r = d_total % n;
#ifdef _OPENMP
    int nt = oracle_threads(threads);
#pragma omp parallel for num_threads(nt) schedule(static)
#endif
    for (int64_t j = 0; j < width; ++j) {
        const int64_t k = k0 + j;
        /* chunk of k: the first r chunks have q + 1 coordinates */
        int64_t c = (k < r * (q + 1)) ? k / (q + 1) : r + (k - r * (q + 1)) / q;
        volatile float acc = updates[c * ld + j];      /* volatile: one rounding per step */
        for (int64_t s = 1; s < n; ++s)
            acc = acc + updates[((c + s) % n) * ld + j];
        if (mean)
            acc = acc / (float)n;
        out[j] = acc;
    }
    return 0;
}
