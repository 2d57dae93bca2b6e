/*
 * CPU oracle for direct sparse convolution.  TEST INFRASTRUCTURE ONLY.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call this file.  It shares no code with the HIP library and is deliberately
 * plain: no blocking, no fusion, no reordering.
 *
 * What it computes (Section 2.1, Eq. (1), extended with batch, stride, zero
 * padding and groups, none of which appear in the equation itself):
 *
 *   out[n,k,y,x] = sum_{c<Cg} sum_{r<R} sum_{s<S}
 *        Wd[k,c,r,s] * in_pad[n, g(k)*Cg + c, y*stride + r, x*stride + s]
 *
 * with g(k) = k / (K/groups), in_pad the input zero-padded by `pad` on all
 * four sides, and Wd the dense weights whose pruned entries are zero.
 * The procedure is the loop nest of Figure 2: per output channel, per stored
 * nonzero (value, pre-lowered offset), per output pixel, one multiply-add of
 * the value with the input shifted by the offset.
 *
 * Pins (tests, not this file): brute-force Eq. (1) on tiny shapes, a library
 * dense convolution at density 1, exact zeros for an empty pattern, linearity
 * in the weights, single-nonzero shift tests, the 1x1 case against a sparse
 * matrix product.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t C, H, W, K, R, S, stride, pad, groups;
} oracle_desc;

static int desc_ok(const oracle_desc *d)
{
    if (!d) return 0;
    if (d->C < 1 || d->H < 1 || d->W < 1 || d->K < 1 || d->R < 1 || d->S < 1) return 0;
    if (d->stride < 1 || d->pad < 0 || d->groups < 1) return 0;
    if (d->C % d->groups || d->K % d->groups) return 0;
    if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S) return 0;
    return 1;
}

int oracle_out_h(const oracle_desc *d) { return (d->H + 2 * d->pad - d->R) / d->stride + 1; }
int oracle_out_w(const oracle_desc *d) { return (d->W + 2 * d->pad - d->S) / d->stride + 1; }

/*
 * CSR of the mode-1 matricised weights (Section 2.1; Figure 2 caption): one
 * row per output channel, column index (c*R + r)*S + s over the group-local
 * input channel c.  Entries equal to zero (either sign) are dropped; every
 * other bit pattern, NaN and Inf included, is kept.  Call with colidx == NULL
 * to count.  Returns nnz, or -1 on a bad descriptor.
 */
int64_t oracle_csr_from_dense(const oracle_desc *d, const float *w,
                              int32_t *rowptr, int32_t *colidx, float *val)
{
    if (!desc_ok(d) || !w) return -1;
    const int64_t ncol = (int64_t)(d->C / d->groups) * d->R * d->S;
    int64_t nnz = 0;
    for (int k = 0; k < d->K; ++k) {
        if (rowptr) rowptr[k] = (int32_t)nnz;
        for (int64_t j = 0; j < ncol; ++j) {
            float v = w[(int64_t)k * ncol + j];
            if (v == 0.0f) continue;
            if (colidx) { colidx[nnz] = (int32_t)j; val[nnz] = v; }
            ++nnz;
        }
    }
    if (rowptr) rowptr[d->K] = (int32_t)nnz;
    return nnz;
}

/*
 * Layout function of Figure 2 for a CHW image, applied to the zero-padded
 * image of one batch element: f(c,r,s) = (c*Hp + r)*Wp + s with
 * Hp = H + 2*pad, Wp = W + 2*pad; c is the absolute input channel
 * g(k)*Cg + c_local of the row's group.
 */
int oracle_lower_offsets(const oracle_desc *d, const int32_t *rowptr,
                         const int32_t *colidx, int32_t *off)
{
    if (!desc_ok(d) || !rowptr || !off) return -1;
    const int Cg = d->C / d->groups, Kg = d->K / d->groups;
    const int Hp = d->H + 2 * d->pad, Wp = d->W + 2 * d->pad;
    for (int k = 0; k < d->K; ++k) {
        const int g = k / Kg;
        for (int32_t j = rowptr[k]; j < rowptr[k + 1]; ++j) {
            const int col = colidx[j];
            const int s = col % d->S;
            const int r = (col / d->S) % d->R;
            const int c = col / (d->S * d->R);
            if (c < 0 || c >= Cg) return -2;
            off[j] = ((g * Cg + c) * Hp + r) * Wp + s;
        }
    }
    return 0;
}

/*
 * The same for an HWC image (channel innermost), the other layout Section 2.1
 * allows: any f with f(c, y+r, x+s) = f(c, y, x) + f(0, r, s) will do.  On the
 * zero-padded HWC image f(c,y,x) = (y*Wp + x)*C + c, so the offset of weight
 * (c, r, s) is (r*Wp + s)*C + g(k)*Cg + c, and moving the output by one row or
 * column moves every read by stride*Wp*C or stride*C elements.
 */
int oracle_lower_offsets_hwc(const oracle_desc *d, const int32_t *rowptr,
                             const int32_t *colidx, int32_t *off)
{
    if (!desc_ok(d) || !rowptr || !off) return -1;
    const int Cg = d->C / d->groups, Kg = d->K / d->groups;
    const int Wp = d->W + 2 * d->pad;
    for (int k = 0; k < d->K; ++k) {
        const int g = k / Kg;
        for (int32_t j = rowptr[k]; j < rowptr[k + 1]; ++j) {
            const int col = colidx[j];
            const int s = col % d->S;
            const int r = (col / d->S) % d->R;
            const int c = col / (d->S * d->R);
            if (c < 0 || c >= Cg) return -2;
            off[j] = (r * Wp + s) * d->C + g * Cg + c;
        }
    }
    return 0;
}

static float *padded_copy(const oracle_desc *d, const float *img)
{
    const int Hp = d->H + 2 * d->pad, Wp = d->W + 2 * d->pad;
    float *p = (float *)calloc((size_t)d->C * Hp * Wp, sizeof(float));
    if (!p) return NULL;
    for (int c = 0; c < d->C; ++c)
        for (int y = 0; y < d->H; ++y)
            memcpy(p + ((size_t)c * Hp + y + d->pad) * Wp + d->pad,
                   img + ((size_t)c * d->H + y) * d->W, sizeof(float) * d->W);
    return p;
}

/*
 * Parity variant.  For every image and output channel, each stored weight
 * slides over the padded image of its input channel (the loop nest of
 * Figure 2): the weight's pre-lowered offset names the top-left corner of
 * the window it multiplies, output pixel (oy, ox) reads the element
 * oy*stride rows and ox*stride columns further.  Every product is formed
 * exactly in fp64 from the two fp32 operands and summed in fp64.
 * out[n][k][oy][ox] receives the sum, absum[n][k][oy][ox] the sum of
 * |products| (the scale of the comparison tolerance).  Either may be NULL.
 */
int oracle_forward_f64(const oracle_desc *d, int32_t N, const int32_t *rowptr,
                       const int32_t *off, const float *val, const float *in,
                       double *out, double *absum)
{
    if (!desc_ok(d) || N < 1 || !rowptr || !in) return -1;
    const int Wp = d->W + 2 * d->pad;
    const int OH = oracle_out_h(d), OW = oracle_out_w(d);
    const size_t plane = (size_t)OH * OW;
    const size_t image_floats = (size_t)d->C * d->H * d->W;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int n = 0; n < N; ++n) {
        float *padded = padded_copy(d, in + (size_t)n * image_floats);
        double *sum = (double *)malloc(sizeof(double) * 2 * plane);
        if (!padded || !sum) { fail = 1; free(padded); free(sum); continue; }
        double *mag = sum + plane;
        for (int k = 0; k < d->K; ++k) {
            for (size_t i = 0; i < 2 * plane; ++i) sum[i] = 0.0;
            for (int32_t e = rowptr[k]; e < rowptr[k + 1]; ++e) {
                const float *window = padded + off[e];
                const double weight = (double)val[e];
                for (int oy = 0; oy < OH; ++oy) {
                    const float *line = window + (size_t)oy * d->stride * Wp;
                    for (int ox = 0; ox < OW; ++ox) {
                        const double prod = weight * (double)line[ox * d->stride];
                        sum[oy * OW + ox] += prod;
                        mag[oy * OW + ox] += fabs(prod);
                    }
                }
            }
            const size_t base = ((size_t)n * d->K + k) * plane;
            if (out) memcpy(out + base, sum, sizeof(double) * plane);
            if (absum) memcpy(absum + base, mag, sizeof(double) * plane);
        }
        free(padded);
        free(sum);
    }
    return fail ? -3 : 0;
}

/*
 * Timed variant: the same walk (image, output channel, stored weight,
 * output pixel) with fp32 multiply-adds in CSR order, the
 * (image, output channel) pairs spread over `nthreads` OpenMP threads
 * (<= 0: all).  Returns the number of threads used, or a negative error.
 */
int oracle_forward_f32(const oracle_desc *d, int32_t N, const int32_t *rowptr,
                       const int32_t *off, const float *val, const float *in,
                       float *out, int nthreads)
{
    if (!desc_ok(d) || N < 1 || !rowptr || !in || !out) return -1;
    const int Wp = d->W + 2 * d->pad;
    const int OH = oracle_out_h(d), OW = oracle_out_w(d);
    const size_t plane = (size_t)OH * OW;
    const size_t image_floats = (size_t)d->C * d->H * d->W;
    float **padded = (float **)calloc((size_t)N, sizeof(float *));
    if (!padded) return -3;
    int used = 1, fail = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
#pragma omp parallel
    {
#ifdef _OPENMP
#pragma omp single
        used = omp_get_num_threads();
#endif
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            padded[n] = padded_copy(d, in + (size_t)n * image_floats);
            if (!padded[n]) fail = 1;
        }
        /* one work item per (image, output channel); the channel's group is implied by its offsets */
#pragma omp for schedule(static)
        for (long item = 0; item < (long)N * d->K; ++item) {
            if (fail) continue;
            const int n = (int)(item / d->K);
            const int k = (int)(item % d->K);
            float *res = out + ((size_t)n * d->K + k) * plane;
            for (size_t i = 0; i < plane; ++i) res[i] = 0.0f;
            for (int32_t e = rowptr[k]; e < rowptr[k + 1]; ++e) {
                const float *window = padded[n] + off[e];
                const float weight = val[e];
                for (int oy = 0; oy < OH; ++oy) {
                    const float *line = window + (size_t)oy * d->stride * Wp;
                    float *dst = res + (size_t)oy * OW;
                    for (int ox = 0; ox < OW; ++ox) dst[ox] += weight * line[ox * d->stride];
                }
            }
        }
    }
    for (int n = 0; n < N; ++n) free(padded[n]);
    free(padded);
    return fail ? -3 : used;
}
