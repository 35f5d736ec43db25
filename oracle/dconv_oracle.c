/*
 * CPU oracle for direct 2D convolution.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain definition of what the two GPU kernels compute,
 * written out as nested loops with fp64 accumulation.  It is used by the
 * tests, by the smoke check and by the benchmark's CPU-baseline leg, and by
 * nothing else; it shares no code with the HIP path.
 *
 * What is computed (paper Sec. 2.2 / Fig. 3a: a C-channel image convolved
 * with a bank of filters, each filter having one FxF window per channel, one
 * output map per filter; Sec. 3: the special case C = 1).  The paper's
 * kernels are exact re-schedulings of this sum (Sec. 4.2: the per-thread
 * accumulator collects the same products, Alg. 2's innermost update), so the
 * oracle is the definition itself, not a replay of the schedule.
 *
 * Readings taken where the paper does not say:
 *   - no filter flip (cross-correlation): in Alg. 2 tap k of a filter row
 *     multiplies the image-row segment starting at offset k, rows taken in
 *     increasing order;
 *   - stride 1, no padding, window anchored top-left: tiles need extra
 *     pixels only to the right and below (Sec. 3.1), one new input row per
 *     downward step;
 *   - a batch dimension (independent images, same filters) is added by the
 *     ABI; the paper has none;
 *   - layouts: in[N][C][H][W], filt[K][C][F][F], out[N][K][Ho][Wo], dense
 *     row-major, Ho = H-F+1, Wo = W-F+1.
 *
 * Letters: K filters of side F (the paper writes K for the side and F for
 * the count).
 *
 * Besides the sum itself every routine can return mag = sum |x*w| per output
 * element, the scale the comparison tolerance is stated in.
 *
 * OpenMP only distributes whole output elements over threads; the order of
 * additions inside one element is always c, then i, then j.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1

static int bad_shape(int64_t N, int64_t C, int64_t H, int64_t W, int64_t K, int64_t F)
{
    return N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || F <= 0 || F > H || F > W;
}

/* One output element: the triple sum over (c, i, j), in fp64. */
static void one_output(const float *in, int64_t C, int64_t H, int64_t W,
                       const float *filt, int64_t F,
                       int64_t n, int64_t k, int64_t y, int64_t x,
                       double *acc_out, double *mag_out)
{
    double acc = 0.0, mag = 0.0;
    for (int64_t c = 0; c < C; ++c) {
        for (int64_t i = 0; i < F; ++i) {
            for (int64_t j = 0; j < F; ++j) {
                double px = (double)in[((n * C + c) * H + (y + i)) * W + (x + j)];
                double wt = (double)filt[((k * C + c) * F + i) * F + j];
                double p = px * wt;   /* exact: 24-bit x 24-bit fits in 53 bits */
                acc += p;
                mag += fabs(p);
            }
        }
    }
    *acc_out = acc;
    *mag_out = mag;
}

/*
 * General case.  Any of out32 / out64 / mag may be NULL.  threads <= 0 means
 * "all the cores OpenMP sees".  Returns the number of threads used through
 * *threads_used when that pointer is not NULL.
 */
int dconv_oracle_general(const float *in, int64_t N, int64_t C, int64_t H, int64_t W,
                         const float *filt, int64_t K, int64_t F,
                         float *out32, double *out64, double *mag,
                         int threads, int *threads_used)
{
    if (!in || !filt || bad_shape(N, C, H, W, K, F)) return ORACLE_BAD_ARG;
    const int64_t Ho = H - F + 1, Wo = W - F + 1;
    const int64_t rows = N * K * Ho;
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    used = threads;
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t y = r % Ho;
        const int64_t k = (r / Ho) % K;
        const int64_t n = r / (Ho * K);
        for (int64_t x = 0; x < Wo; ++x) {
            double acc, m;
            one_output(in, C, H, W, filt, F, n, k, y, x, &acc, &m);
            const int64_t o = r * Wo + x;
            if (out32) out32[o] = (float)acc;
            if (out64) out64[o] = acc;
            if (mag) mag[o] = m;
        }
    }
    if (threads_used) *threads_used = used;
    return ORACLE_OK;
}

/*
 * Special case (paper Sec. 3): one image, one channel.  Written out on its
 * own rather than forwarded, so that the two definitions check each other.
 * img[H][W], filt[K][F][F], out[K][Ho][Wo].
 */
int dconv_oracle_single_channel(const float *img, int64_t H, int64_t W,
                                const float *filt, int64_t K, int64_t F,
                                float *out32, double *out64, double *mag,
                                int threads, int *threads_used)
{
    if (!img || !filt || bad_shape(1, 1, H, W, K, F)) return ORACLE_BAD_ARG;
    const int64_t Ho = H - F + 1, Wo = W - F + 1;
    const int64_t rows = K * Ho;
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    used = threads;
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
    for (int64_t r = 0; r < rows; ++r) {
        const int64_t k = r / Ho, y = r % Ho;
        for (int64_t x = 0; x < Wo; ++x) {
            double acc = 0.0, m = 0.0;
            for (int64_t i = 0; i < F; ++i) {
                for (int64_t j = 0; j < F; ++j) {
                    double p = (double)img[(y + i) * W + (x + j)] *
                               (double)filt[(k * F + i) * F + j];
                    acc += p;
                    m += fabs(p);
                }
            }
            const int64_t o = r * Wo + x;
            if (out32) out32[o] = (float)acc;
            if (out64) out64[o] = acc;
            if (mag) mag[o] = m;
        }
    }
    if (threads_used) *threads_used = used;
    return ORACLE_OK;
}

/*
 * The same sums for a list of output elements only, each named by its flat
 * index into out[N][K][Ho][Wo].  Lets a test check sampled elements of an
 * output too large to compute whole on the CPU.
 */
int dconv_oracle_general_at(const float *in, int64_t N, int64_t C, int64_t H, int64_t W,
                            const float *filt, int64_t K, int64_t F,
                            const int64_t *flat_idx, int64_t count,
                            double *acc, double *mag)
{
    if (!in || !filt || !flat_idx || !acc || !mag || count < 0 ||
        bad_shape(N, C, H, W, K, F))
        return ORACLE_BAD_ARG;
    const int64_t Ho = H - F + 1, Wo = W - F + 1;
    const int64_t total = N * K * Ho * Wo;
    for (int64_t q = 0; q < count; ++q)
        if (flat_idx[q] < 0 || flat_idx[q] >= total) return ORACLE_BAD_ARG;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t q = 0; q < count; ++q) {
        int64_t o = flat_idx[q];
        const int64_t x = o % Wo; o /= Wo;
        const int64_t y = o % Ho; o /= Ho;
        const int64_t k = o % K;
        const int64_t n = o / K;
        one_output(in, C, H, W, filt, F, n, k, y, x, &acc[q], &mag[q]);
    }
    return ORACLE_OK;
}

int dconv_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
