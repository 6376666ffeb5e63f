/*
 * CPU oracle for the strided-kernel (SK) network layers.  TEST INFRASTRUCTURE ONLY:
 * it exists so that tests, the smoke check and the benchmark's cpu_baseline leg can
 * compare the GPU library against a plain implementation.  The product never calls it.
 *
 * Everything is fp64, NCHW, contiguous, plain nested loops.  Each output element is
 * accumulated in the order (c, i, j) = (input map, kernel row, kernel column), the K order
 * of the paper's GEMM view (Section 5.5, "Convolution Methods").  The OpenMP pragmas only
 * distribute independent output rows over threads; they do not change any sum.
 *
 * Conventions the paper leaves open and that are fixed here (parity unpinned by the paper; the
 * oracle and the GPU library simply have to agree): which mirror variant pads the border, that
 * every conv has one bias per output map, the max-pool tie-break (first maximum in row-major
 * tap order), ReLU'(0) = 0, and the SGD update rule.  Everything else is pinned by
 * tests/test_oracle_pins.py against the paper's tables, the sliding-window definition evaluated
 * by brute force, closed forms, library routines and finite differences.
 *
 * Notation follows Section 1.6 (Terminology): f_in/f_out feature maps, w map size, k kernel
 * size, d kernel stride (= dilation), s layer stride, n minibatch.
 */
#include <stddef.h>
#include <stdint.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- threads: how many the parallel loops below use, and a way to set that number (the benchmark
 *      reports the oracle's speed with the count it really ran on, and once on a single thread).
 *      No arithmetic depends on it. ---- */
int osk_get_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void osk_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- border mirroring (Section 1.3: the image is extended by mirroring so that every
 *      pixel has its full context).  mode 0: reflect without repeating the edge sample,
 *      mode 1: symmetric (edge sample repeated). ---- */
static long mirror_index(long t, long len, int mode)
{
    /* fold t into [0, len) */
    if (len == 1) return 0;
    if (mode == 0) {
        long period = 2 * (len - 1);
        t %= period;
        if (t < 0) t += period;
        return t < len ? t : period - t;
    } else {
        long period = 2 * len;
        t %= period;
        if (t < 0) t += period;
        return t < len ? t : period - 1 - t;
    }
}

void osk_mirror_pad(const double *in, long planes, long h, long w,
                    long top, long left, long bottom, long right, int mode, double *out)
{
    long ho = h + top + bottom, wo = w + left + right;
    for (long p = 0; p < planes; ++p)
        for (long y = 0; y < ho; ++y)
            for (long x = 0; x < wo; ++x)
                out[(p * ho + y) * wo + x] =
                    in[(p * h + mirror_index(y - top, h, mode)) * w + mirror_index(x - left, w, mode)];
}

/* ---- SK convolution (Section 5.2.1 "SK Layers"; Algorithm 1: s = 1, p = 0):
 *      Y[o,y,x] = b[o] + sum_{c,i,j} W[o,c,i,j] * X[c, y + i*d, x + j*d]
 *      output size w_out = w_in - (k-1)*d.  Cross-correlation (no kernel flip). ---- */
void osk_conv_sk(const double *x, long n, long f_in, long h, long w,
                 const double *wgt, const double *bias, long f_out, long k, long d,
                 int relu, double *y)
{
    long ho = h - (k - 1) * d, wo = w - (k - 1) * d;
    for (long b = 0; b < n; ++b) {
#pragma omp parallel for collapse(2) schedule(static)
        for (long o = 0; o < f_out; ++o)
            for (long yy = 0; yy < ho; ++yy) {
                double *row = y + ((b * f_out + o) * ho + yy) * wo;
                for (long xx = 0; xx < wo; ++xx) row[xx] = bias ? bias[o] : 0.0;
                for (long c = 0; c < f_in; ++c)
                    for (long i = 0; i < k; ++i)
                        for (long j = 0; j < k; ++j) {
                            double wv = wgt[((o * f_in + c) * k + i) * k + j];
                            const double *src = x + ((b * f_in + c) * h + yy + i * d) * w + j * d;
                            for (long xx = 0; xx < wo; ++xx) row[xx] += wv * src[xx];
                        }
                if (relu)
                    for (long xx = 0; xx < wo; ++xx) row[xx] = row[xx] > 0.0 ? row[xx] : 0.0;
            }
    }
}

/* ---- data gradient of the SK convolution: exact adjoint of the map X -> Y above.
 *      dX[c,u,v] = sum_{o,i,j} W[o,c,i,j] * dY[o, u - i*d, v - j*d]  (terms outside dY dropped) ---- */
void osk_conv_sk_bwd_data(const double *dy, long n, long f_in, long h, long w,
                          const double *wgt, long f_out, long k, long d, double *dx)
{
    long ho = h - (k - 1) * d, wo = w - (k - 1) * d;
    for (long b = 0; b < n; ++b) {
#pragma omp parallel for collapse(2) schedule(static)
        for (long c = 0; c < f_in; ++c)
            for (long u = 0; u < h; ++u) {
                double *row = dx + ((b * f_in + c) * h + u) * w;
                for (long v = 0; v < w; ++v) row[v] = 0.0;
                for (long o = 0; o < f_out; ++o)
                    for (long i = 0; i < k; ++i) {
                        long yy = u - i * d;
                        if (yy < 0 || yy >= ho) continue;
                        for (long j = 0; j < k; ++j) {
                            double wv = wgt[((o * f_in + c) * k + i) * k + j];
                            const double *src = dy + ((b * f_out + o) * ho + yy) * wo;
                            for (long v = 0; v < w; ++v) {
                                long xx = v - j * d;
                                if (xx >= 0 && xx < wo) row[v] += wv * src[xx];
                            }
                        }
                    }
            }
    }
}

/* ---- weight and bias gradient:
 *      dW[o,c,i,j] = sum_{n,y,x} dY[o,y,x] * X[c, y + i*d, x + j*d],  db[o] = sum_{n,y,x} dY[o,y,x] ---- */
void osk_conv_sk_bwd_weights(const double *x, const double *dy, long n, long f_in, long h, long w,
                             long f_out, long k, long d, double *dw, double *db)
{
    long ho = h - (k - 1) * d, wo = w - (k - 1) * d;
#pragma omp parallel for collapse(2) schedule(static)
    for (long o = 0; o < f_out; ++o)
        for (long c = 0; c < f_in; ++c)
            for (long i = 0; i < k; ++i)
                for (long j = 0; j < k; ++j) {
                    double acc = 0.0;
                    for (long b = 0; b < n; ++b)
                        for (long yy = 0; yy < ho; ++yy) {
                            const double *g = dy + ((b * f_out + o) * ho + yy) * wo;
                            const double *src = x + ((b * f_in + c) * h + yy + i * d) * w + j * d;
                            for (long xx = 0; xx < wo; ++xx) acc += g[xx] * src[xx];
                        }
                    dw[((o * f_in + c) * k + i) * k + j] = acc;
                }
    if (db)
        for (long o = 0; o < f_out; ++o) {
            double acc = 0.0;
            for (long b = 0; b < n; ++b)
                for (long q = 0; q < ho * wo; ++q) acc += dy[(b * f_out + o) * ho * wo + q];
            db[o] = acc;
        }
}

/* ---- max pooling with kernel stride d and layer stride s (Section 5.2.1; Algorithm 1 turns
 *      a k = s down-sampling pool into s = 1 with kernel stride d; the U-Net keeps s = k, d = 1):
 *      Y[c,y,x] = max_{i,j<k} X[c, s*y + i*d, s*x + j*d],  w_out = (w_in - (k-1)*d - 1)/s + 1.
 *      Taps are scanned row-major and replaced only on strictly greater: the first maximum
 *      wins.  argmax = flat offset of the winning sample inside its input plane. ---- */
void osk_maxpool_sk(const double *x, long planes, long h, long w, long k, long d, long s,
                    double *y, int32_t *argmax)
{
    long ho = (h - (k - 1) * d - 1) / s + 1, wo = (w - (k - 1) * d - 1) / s + 1;
#pragma omp parallel for schedule(static)
    for (long p = 0; p < planes; ++p)
        for (long yy = 0; yy < ho; ++yy)
            for (long xx = 0; xx < wo; ++xx) {
                long best = (s * yy) * w + s * xx;
                double bv = x[p * h * w + best];
                for (long i = 0; i < k; ++i)
                    for (long j = 0; j < k; ++j) {
                        long at = (s * yy + i * d) * w + s * xx + j * d;
                        double v = x[p * h * w + at];
                        if (v > bv) { bv = v; best = at; }
                    }
                y[(p * ho + yy) * wo + xx] = bv;
                if (argmax) argmax[(p * ho + yy) * wo + xx] = (int32_t)best;
            }
}

/* pool backward: every output sends its gradient to the recorded winner */
void osk_maxpool_bwd(const double *dy, const int32_t *argmax, long planes, long h, long w,
                     long ho, long wo, double *dx)
{
    for (long q = 0; q < planes * h * w; ++q) dx[q] = 0.0;
    for (long p = 0; p < planes; ++p)
        for (long q = 0; q < ho * wo; ++q)
            dx[p * h * w + argmax[p * ho * wo + q]] += dy[p * ho * wo + q];
}

/* ReLU backward: gradient passes where the (post-ReLU) output is strictly positive */
void osk_relu_bwd(const double *y, const double *dy, long count, double *dx)
{
    for (long q = 0; q < count; ++q) dx[q] = y[q] > 0.0 ? dy[q] : 0.0;
}

/* ---- per-pixel softmax over the class maps: p_c = exp(z_c - m) / sum_j exp(z_j - m) ---- */
void osk_softmax(const double *z, long n, long classes, long hw, double *p)
{
    for (long b = 0; b < n; ++b)
        for (long q = 0; q < hw; ++q) {
            double m = z[(b * classes) * hw + q];
            for (long c = 1; c < classes; ++c) {
                double v = z[(b * classes + c) * hw + q];
                if (v > m) m = v;
            }
            double sum = 0.0;
            for (long c = 0; c < classes; ++c) sum += exp(z[(b * classes + c) * hw + q] - m);
            for (long c = 0; c < classes; ++c)
                p[(b * classes + c) * hw + q] = exp(z[(b * classes + c) * hw + q] - m) / sum;
        }
}

/* ---- softmax loss (Section 4.3: the loss is accumulated over all error pixels and then
 *      normalised): L = -(1/P) sum log p_label, dz = (p - onehot)/P over the pixels that carry a
 *      label in 0..classes-1; a pixel with any other label value (-1 by convention) is masked out
 *      of the error map (Section 4.2's label masking): it adds nothing to the loss, its gradient is
 *      zero, and P counts the unmasked pixels only (P = n*h*w without masking). ---- */
double osk_softmax_loss(const double *z, const int32_t *labels, long n, long classes, long hw,
                        double *dz)
{
    double total = 0.0;
    long kept = 0;
    for (long q = 0; q < n * hw; ++q)
        if (labels[q] >= 0 && labels[q] < classes) ++kept;
    const double P = kept > 0 ? (double)kept : 1.0;
    for (long b = 0; b < n; ++b)
        for (long q = 0; q < hw; ++q) {
            long lab = labels[b * hw + q];
            if (lab < 0 || lab >= classes) {
                if (dz)
                    for (long c = 0; c < classes; ++c) dz[(b * classes + c) * hw + q] = 0.0;
                continue;
            }
            double m = z[(b * classes) * hw + q];
            for (long c = 1; c < classes; ++c) {
                double v = z[(b * classes + c) * hw + q];
                if (v > m) m = v;
            }
            double sum = 0.0;
            for (long c = 0; c < classes; ++c) sum += exp(z[(b * classes + c) * hw + q] - m);
            total -= z[(b * classes + lab) * hw + q] - m - log(sum);
            if (dz)
                for (long c = 0; c < classes; ++c) {
                    double pc = exp(z[(b * classes + c) * hw + q] - m) / sum;
                    dz[(b * classes + c) * hw + q] = (pc - (c == lab ? 1.0 : 0.0)) / P;
                }
        }
    return total / P;
}

/* ---- 2x2, stride-2 up-convolution (U-Net expanding step, Section 3.4): every input pixel
 *      fills one 2x2 output block.  General learned form
 *      Y[o, 2y+a, 2x+b] = bias[o] + sum_c W[c,o,a,b] * X[c,y,x];
 *      the paper's fixed nearest-neighbour, one-map-per-group version is W[c,o,a,b] = (c == o). ---- */
void osk_upconv2x2(const double *x, long n, long f_in, long h, long w,
                   const double *wgt, const double *bias, long f_out, double *y)
{
    long ho = 2 * h, wo = 2 * w;
    for (long b = 0; b < n; ++b) {
#pragma omp parallel for schedule(static)
        for (long o = 0; o < f_out; ++o)
            for (long yy = 0; yy < h; ++yy)
                for (long xx = 0; xx < w; ++xx)
                    for (long a = 0; a < 2; ++a)
                        for (long bb = 0; bb < 2; ++bb) {
                            double acc = bias ? bias[o] : 0.0;
                            for (long c = 0; c < f_in; ++c)
                                acc += wgt[((c * f_out + o) * 2 + a) * 2 + bb] *
                                       x[((b * f_in + c) * h + yy) * w + xx];
                            y[((b * f_out + o) * ho + 2 * yy + a) * wo + 2 * xx + bb] = acc;
                        }
    }
}

/* ---- MergeCrop (Section 5.3.1): output = all maps of A, then all maps of B centre-cropped
 *      to A's size; w_B >= w_A, offset floor((w_B - w_A)/2). ---- */
void osk_mergecrop(const double *a, long n, long fa, long ha, long wa,
                   const double *bsrc, long fb, long hb, long wb, double *out)
{
    long oy = (hb - ha) / 2, ox = (wb - wa) / 2, fo = fa + fb;
    for (long b = 0; b < n; ++b) {
        for (long c = 0; c < fa; ++c)
            for (long q = 0; q < ha * wa; ++q)
                out[(b * fo + c) * ha * wa + q] = a[(b * fa + c) * ha * wa + q];
        for (long c = 0; c < fb; ++c)
            for (long yy = 0; yy < ha; ++yy)
                for (long xx = 0; xx < wa; ++xx)
                    out[((b * fo + fa + c) * ha + yy) * wa + xx] =
                        bsrc[((b * fb + c) * hb + yy + oy) * wb + xx + ox];
    }
}

/* ---- SGD with momentum and weight decay: g = dW + lambda*W; V = mu*V + lr*g; W = W - V ---- */
void osk_sgd(double *wgt, const double *dw, double *vel, long count,
             double lr, double momentum, double weight_decay)
{
    for (long q = 0; q < count; ++q) {
        double g = dw[q] + weight_decay * wgt[q];
        double v = (vel ? momentum * vel[q] : 0.0) + lr * g;
        if (vel) vel[q] = v;
        wgt[q] -= v;
    }
}
