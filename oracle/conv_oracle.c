/*
 * CPU oracle for the forward 2-D convolution operator.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call, link or import this file; it shares no code
 * with the HIP kernels.
 *
 * What it computes is the plain definition of the operator the paper optimises
 * (Section 2.3 "State space": problem parameters N, C_in, C_out, K_h, K_w, H, W, Stride,
 * Padding; Section 2.2 "Halide compiler": the sample algorithm multiplies filter(r)
 * by in(x + r - 1), i.e. cross-correlation without a filter flip, with the padding
 * shift subtracted from the input coordinate).  Widened, as the build's target asks,
 * to separate h/w stride, symmetric zero padding and dilation:
 *
 *   y[n,k,p,q] = sum_{c<C} sum_{r<R} sum_{s<S}
 *                x[n, c, p*stride_h - pad_h + r*dil_h, q*stride_w - pad_w + s*dil_w] * w[k,c,r,s]
 *
 * with taps outside the image contributing zero, and
 *   P = floor((H + 2*pad_h - dil_h*(R-1) - 1) / stride_h) + 1   (Q alike).
 *
 * Seven nested loops in the order n,k,p,q,c,r,s.  Inputs are fp32, promoted to fp64;
 * every product and the running sum are fp64; no blocking, no re-association.
 * Next to y it returns the normaliser D = sum |x*w| over the same taps, which the
 * parity tests divide errors by.
 *
 * Pins (tests/test_oracle_conv.py): scatter-form and im2col brute force on tiny
 * shapes, delta-kernel identities, all-ones tap-count closed form, linearity,
 * 1x1 == matrix product, full-window == dot product, translation equivariance,
 * output-shape values of the ResNet layers.
 *
 * Threads: OpenMP over the (n,k) pairs only.  Every output is still summed by one
 * thread in the c,r,s order above, so the thread count changes no result bit.
 */
#include <stdint.h>
#include <stddef.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t n, c, h, w;
    int32_t k, r, s;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} oracle_conv_shape;

/* floor division for possibly negative numerators, positive denominators */
static int64_t floordiv(int64_t a, int64_t b)
{
    int64_t q = a / b;
    if ((a % b != 0) && ((a < 0) != (b < 0))) q -= 1;
    return q;
}

/* Output extent along one axis; returns <= 0 when the window does not fit. */
int64_t oracle_out_extent(int64_t in, int64_t pad, int64_t dil, int64_t win, int64_t stride)
{
    int64_t span = in + 2 * pad - dil * (win - 1) - 1;
    if (span < 0) return 0;
    return floordiv(span, stride) + 1;
}

int oracle_conv_out_shape(const oracle_conv_shape *d, int64_t *p, int64_t *q)
{
    if (!d || d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0 || d->k <= 0 || d->r <= 0 ||
        d->s <= 0 || d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0 ||
        d->dil_h <= 0 || d->dil_w <= 0)
        return -1;
    *p = oracle_out_extent(d->h, d->pad_h, d->dil_h, d->r, d->stride_h);
    *q = oracle_out_extent(d->w, d->pad_w, d->dil_w, d->s, d->stride_w);
    return (*p > 0 && *q > 0) ? 0 : -1;
}

/* One output element: the three inner loops c,r,s. */
static void one_output(const oracle_conv_shape *d, const float *x, const float *w,
                       int64_t n, int64_t k, int64_t p, int64_t q, double *y, double *dn)
{
    double acc = 0.0, mag = 0.0;
    for (int64_t c = 0; c < d->c; ++c) {
        for (int64_t r = 0; r < d->r; ++r) {
            for (int64_t s = 0; s < d->s; ++s) {
                int64_t ih = p * d->stride_h - d->pad_h + r * d->dil_h;
                int64_t iw = q * d->stride_w - d->pad_w + s * d->dil_w;
                if (ih < 0 || ih >= d->h || iw < 0 || iw >= d->w) continue; /* zero padding */
                double xv = (double)x[((n * d->c + c) * d->h + ih) * d->w + iw];
                double wv = (double)w[((k * d->c + c) * d->r + r) * d->s + s];
                double t = xv * wv;
                acc += t;
                mag += fabs(t);
            }
        }
    }
    *y = acc;
    *dn = mag;
}

/*
 * Full tensor.  x: [N][C][H][W] fp32, w: [K][C][R][S] fp32 (host pointers, read only).
 * y64 / y32 / dnorm: [N][K][P][Q]; any of them may be NULL.  threads <= 0 means "all".
 * Returns the thread count actually used, or -1 on a bad shape.
 */
int oracle_conv2d_fwd(const oracle_conv_shape *d, const float *x, const float *w, double *y64,
                      float *y32, double *dnorm, int threads)
{
    int64_t P, Q;
    if (oracle_conv_out_shape(d, &P, &Q) != 0 || !x || !w) return -1;
    int used = 1;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    used = threads;
#else
    (void)threads;
#endif
    int64_t NK = (int64_t)d->n * d->k;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(threads)
#endif
    for (int64_t nk = 0; nk < NK; ++nk) {
        int64_t n = nk / d->k, k = nk % d->k;
        for (int64_t p = 0; p < P; ++p) {
            for (int64_t q = 0; q < Q; ++q) {
                double yv, dv;
                one_output(d, x, w, n, k, p, q, &yv, &dv);
                int64_t o = ((n * d->k + k) * P + p) * Q + q;
                if (y64) y64[o] = yv;
                if (y32) y32[o] = (float)yv;
                if (dnorm) dnorm[o] = dv;
            }
        }
    }
    return used;
}

/*
 * Sampled outputs: idx holds flat offsets into [N][K][P][Q]; y64[i], dnorm[i] receive the
 * value and normaliser of output idx[i].  Used where the full tensor is too slow.
 */
int oracle_conv2d_sampled(const oracle_conv_shape *d, const float *x, const float *w,
                          const int64_t *idx, int64_t count, double *y64, double *dnorm)
{
    int64_t P, Q;
    if (oracle_conv_out_shape(d, &P, &Q) != 0 || !x || !w || !idx) return -1;
    int64_t total = (int64_t)d->n * d->k * P * Q;
    for (int64_t i = 0; i < count; ++i) {
        int64_t o = idx[i];
        if (o < 0 || o >= total) return -2;
        int64_t q = o % Q, p = (o / Q) % P, k = (o / (Q * P)) % d->k, n = o / (Q * P * d->k);
        double yv, dv;
        one_output(d, x, w, n, k, p, q, &yv, &dv);
        if (y64) y64[i] = yv;
        if (dnorm) dnorm[i] = dv;
    }
    return 0;
}
