/*
 * conv_ref.c -- CPU oracle for the forward pass of a dense 2-D convolution layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is checked against.  Nothing in the product path may include, link or
 * call it; only tests, the smoke check and the benchmark's cpu_baseline leg do.
 * It shares no code, headers, tables or helpers with the HIP implementation.
 *
 * What it computes (paper: Section 3, Algorithm 1, the single
 * multiply-accumulate statement inside six nested loops), extended with a batch
 * dimension and symmetric zero padding:
 *
 *   P = floor((H + 2*pad - R) / stride) + 1,   Q = floor((W + 2*pad - S) / stride) + 1
 *   out[n][k][p][q] = sum over c, r, s of
 *        in[n][c][p*stride + r - pad][q*stride + s - pad] * w[k][c][r][s]
 *
 * where a tap that falls outside the image contributes nothing.  The filter is not
 * flipped (the paper's statement indexes input and filter with the same m, n).
 * Paper index names -> names here: i -> c (input channel), j -> k (output channel),
 * k -> q (output column), l -> p (output row), m -> s (filter column),
 * n -> r (filter row), s -> stride.  Indices are 0-based.
 *
 * Precision: inputs are fp32 as handed to the GPU; every value is widened to
 * double, each product of two widened fp32 values is exact in double, and the sum
 * is accumulated in double in the fixed order c, r, s.  No blocking, fusion or
 * reordering beyond the definition.
 *
 * Pins (see the CPU tests): shape example of the paper's Figure 2 caption,
 * an independent fp64 im2col + matrix product, the loop order of Algorithm 2,
 * 1x1 convolution == matrix product, delta filter == shifted crop, closed-form
 * tap counts for all-ones tensors, explicit zero padding, stride subsampling,
 * linearity, batch / output-channel independence.  Nothing here is unpinned.
 *
 * Layouts (row-major, last index fastest): in  [N][C][H][W], w [K][C][R][S],
 * out [N][K][P][Q].
 */
#include <stddef.h>
#include <stdint.h>

/* Output extent along one dimension; <= 0 means the filter does not fit. */
int conv_ref_out_dim(int in_extent, int filter_extent, int stride, int pad)
{
    int span = in_extent + 2 * pad - filter_extent;
    if (in_extent <= 0 || filter_extent <= 0 || stride <= 0 || pad < 0 || span < 0)
        return 0;
    return span / stride + 1;
}

static int check_dims(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                      int *P, int *Q)
{
    if (N <= 0 || C <= 0 || K <= 0)
        return -1;
    *P = conv_ref_out_dim(H, R, stride, pad);
    *Q = conv_ref_out_dim(W, S, stride, pad);
    if (*P <= 0 || *Q <= 0)
        return -1;
    return 0;
}

/* One output element: the innermost three loops (c, r, s) of the definition. */
static double one_output(const float *in, const float *w, int n, int k, int p, int q,
                         int C, int H, int W, int R, int S, int stride, int pad)
{
    double acc = 0.0;
    for (int c = 0; c < C; ++c) {
        for (int r = 0; r < R; ++r) {
            int ih = p * stride + r - pad;
            if (ih < 0 || ih >= H)
                continue;
            for (int s = 0; s < S; ++s) {
                int iw = q * stride + s - pad;
                if (iw < 0 || iw >= W)
                    continue;
                double x = (double)in[(((size_t)n * C + c) * H + ih) * W + iw];
                double f = (double)w[(((size_t)k * C + c) * R + r) * S + s];
                acc += x * f;
            }
        }
    }
    return acc;
}

/*
 * Full forward pass.  out must hold N*K*P*Q doubles.  Returns 0, or -1 when the
 * dimensions do not describe a convolution.  The (n, k) planes are independent, so
 * the optional OpenMP pragma splits them over threads without changing any sum.
 */
int conv_ref_forward(const float *in, const float *w, double *out,
                     int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    int P, Q;
    if (check_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q))
        return -1;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static)
#endif
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q)
                    out[(((size_t)n * K + k) * P + p) * Q + q] =
                        one_output(in, w, n, k, p, q, C, H, W, R, S, stride, pad);
    return 0;
}

/*
 * The same definition evaluated only at listed outputs: idx holds npts quadruples
 * (n, k, p, q); out receives npts doubles.  Used to check full-size layers on a
 * sample.  Returns -1 on bad dimensions, -2 if an index is out of range.
 */
int conv_ref_forward_points(const float *in, const float *w, const int32_t *idx, double *out,
                            size_t npts,
                            int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    int P, Q;
    if (check_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q))
        return -1;
    int bad = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) reduction(| : bad)
#endif
    for (size_t t = 0; t < npts; ++t) {
        int n = idx[4 * t + 0], k = idx[4 * t + 1], p = idx[4 * t + 2], q = idx[4 * t + 3];
        if (n < 0 || n >= N || k < 0 || k >= K || p < 0 || p >= P || q < 0 || q >= Q) {
            bad |= 1;
            continue;
        }
        out[t] = one_output(in, w, n, k, p, q, C, H, W, R, S, stride, pad);
    }
    return bad ? -2 : 0;
}

/*
 * Second evaluation order, for self-checking only (paper: Section 3.1.2,
 * Algorithm 2): per image the loops run output row, filter
 * row, filter column, input channel, output column, output channel, and every
 * statement adds into out, which therefore starts at zero.  On inputs whose
 * partial sums are all exactly representable this must equal conv_ref_forward
 * bit for bit (Section 3: the loops may run in any order).  Serial on purpose.
 */
int conv_ref_forward_reordered(const float *in, const float *w, double *out,
                               int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    int P, Q;
    if (check_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q))
        return -1;
    size_t total = (size_t)N * K * P * Q;
    for (size_t t = 0; t < total; ++t)
        out[t] = 0.0;
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int r = 0; r < R; ++r) {
                int ih = p * stride + r - pad;
                if (ih < 0 || ih >= H)
                    continue;
                for (int s = 0; s < S; ++s)
                    for (int c = 0; c < C; ++c)
                        for (int q = 0; q < Q; ++q) {
                            int iw = q * stride + s - pad;
                            if (iw < 0 || iw >= W)
                                continue;
                            double x = (double)in[(((size_t)n * C + c) * H + ih) * W + iw];
                            for (int k = 0; k < K; ++k)
                                out[(((size_t)n * K + k) * P + p) * Q + q] +=
                                    x * (double)w[(((size_t)k * C + c) * R + r) * S + s];
                        }
            }
    return 0;
}

/*
 * Data gradient of the layer (the backward pass with respect to the input image, which
 * the paper's closing section names as a direction; not an algorithm of the paper): the
 * adjoint of the forward map in its input argument, i.e. every product of the
 * definition above, scattered back to the input element it read:
 *
 *   dx[n][c][h][w] = sum over k, r, s of  dy[n][k][p][q] * w[k][c][r][s]
 *        for the (p, q) with p*stride + r - pad == h and q*stride + s - pad == w,
 *        0 <= p < P, 0 <= q < Q  (no such p or q: the term is absent).
 *
 * Written as a gather: for each dx element the loops k, r, s in that order, fp64
 * accumulation.  Pinned by the adjoint identity <dy, forward(x, w)> == <dgrad(dy, w), x>
 * (exact on integers), delta filters, and the stride-1 identity with a forward pass
 * over the flipped, transposed filter.
 */
int conv_ref_dgrad(const float *dy, const float *w, double *dx,
                   int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    int P, Q;
    if (check_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return -1;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static)
#endif
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int x = 0; x < W; ++x) {
                    double acc = 0.0;
                    for (int k = 0; k < K; ++k)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                const int ph = h + pad - r, qw = x + pad - s;
                                if (ph < 0 || qw < 0 || ph % stride || qw % stride) continue;
                                const int p = ph / stride, q = qw / stride;
                                if (p >= P || q >= Q) continue;
                                acc += (double)dy[(((size_t)n * K + k) * P + p) * Q + q] *
                                       (double)w[(((size_t)k * C + c) * R + r) * S + s];
                            }
                    dx[(((size_t)n * C + c) * H + h) * W + x] = acc;
                }
    return 0;
}

/*
 * Weight gradient of the layer (the backward pass with respect to the filter, named in the
 * paper's closing section; not an algorithm of the paper): the adjoint of the forward map
 * in its filter argument, i.e. every product of the definition, collected per filter
 * element:
 *
 *   dw[k][c][r][s] = sum over n, p, q of
 *        dy[n][k][p][q] * x[n][c][p*stride + r - pad][q*stride + s - pad]
 *
 * (taps outside the image absent).  Loops n, p, q in that order per dw element, fp64
 * accumulation.  Pinned by <dy, forward(x, w)> == <wgrad(x, dy), w> (exact on
 * integers), single-element filters, and float64 autograd.
 */
int conv_ref_wgrad(const float *x, const float *dy, double *dw,
                   int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    int P, Q;
    if (check_dims(N, C, H, W, K, R, S, stride, pad, &P, &Q)) return -1;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) schedule(static)
#endif
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < P; ++p)
                            for (int q = 0; q < Q; ++q) {
                                const int ih = p * stride + r - pad, iw = q * stride + s - pad;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += (double)dy[(((size_t)n * K + k) * P + p) * Q + q] *
                                       (double)x[(((size_t)n * C + c) * H + ih) * W + iw];
                            }
                    dw[(((size_t)k * C + c) * R + r) * S + s] = acc;
                }
    return 0;
}

/* Number of threads conv_ref_forward will use (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int conv_ref_threads(void) { return omp_get_max_threads(); }
#else
int conv_ref_threads(void) { return 1; }
#endif
