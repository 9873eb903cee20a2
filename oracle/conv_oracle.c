/*
 * conv_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU definition of the forward 2-D convolution with the
 * fused bias + activation epilogue, in fp64.  It exists only so that the tests, the smoke check
 * and the cpu_baseline leg of the benchmark have something independent to compare the GPU
 * library against.  Nothing in the GPU library includes, links or calls this file, and this
 * file includes nothing from the GPU library.
 *
 * What it follows (MIOpen paper, arXiv 1910.00078):
 *   - Tensor roles W[K,C,Y,X], I[N,C,H,W], O[N,K,H^,W^]: Fig. 2 (Sec. IV-A "Composable Kernels").
 *   - The convolution descriptor carries striding, dilation and padding: Sec. IV-A (find step).
 *   - Grouped convolution = split channels into groups, convolve each with its own filters,
 *     stack the results: Sec. IV-A "Grouped convolutions".
 *   - Convolution followed by a bias addition and ReLU, with no intermediate written out:
 *     Sec. V (Fusion API).
 *   - Conv + bias + inference batch-norm + activation (the CBNA row): Tables I/II, with the
 *     normalisation of Sec. IV-B (spatial mode: one mean/variance/scale/shift per channel).
 *
 * The paper never prints the convolution formula.  The reading used here (the one every
 * framework the paper serves uses) is cross-correlation -- no filter flip -- with zero padding
 * applied symmetrically, floor division in the output-size rule, tap spacing = dilation:
 *
 *   Ho = floor((H + 2*pad_h - dil_h*(R-1) - 1) / stride_h) + 1          (Wo likewise)
 *   pre[n,k,p,q] = b[k] + sum_{c in group(k)} sum_{r<R} sum_{s<S}
 *                    xz[n, c, p*stride_h - pad_h + r*dil_h, q*stride_w - pad_w + s*dil_w]
 *                    * w[k, c - c0(k), r, s]
 *   xz = x inside [0,H)x[0,W), 0 outside
 *   y = act(pre)       identity | relu max(pre,0) | leaky (pre>0 ? pre : alpha*pre)
 *                      | tanh | logistic 1/(1+exp(-pre))
 *
 * Loops are written in exactly that order: n, k, p, q, then c, r, s.  No tiling, no SIMD
 * intrinsics, no BLAS.  OpenMP splits only the outer (n,k) pairs.
 *
 * Pins: every function here is pinned by tests/test_oracle_pins.py (hand-worked examples under
 * tests/golden/, closed forms, identities, scipy/numpy library routines, im2col brute force).
 */
#include <math.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ACT_IDENTITY = 0, ACT_RELU = 1, ACT_LEAKY_RELU = 2, ACT_TANH = 3, ACT_LOGISTIC = 4 };

static double apply_act(double v, int act, double alpha)
{
    switch (act) {
    case ACT_RELU:       return v > 0.0 ? v : 0.0;
    case ACT_LEAKY_RELU: return v > 0.0 ? v : alpha * v;
    case ACT_TANH:       return tanh(v);
    case ACT_LOGISTIC:   return 1.0 / (1.0 + exp(-v));
    default:             return v;
    }
}

/* Output extent along one axis; <= 0 means the filter does not fit even once. */
int conv_oracle_out_extent(int in, int filt, int pad, int stride, int dil)
{
    if (in < 1 || filt < 1 || pad < 0 || stride < 1 || dil < 1) return 0;
    int span = in + 2 * pad - dil * (filt - 1) - 1;
    if (span < 0) return 0;
    return span / stride + 1;
}

int conv_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One output element, pre-activation, without bias. */
static double conv_point(const double *x, const double *w,
                         int C, int H, int W, int K, int R, int S,
                         int pad_h, int pad_w, int stride_h, int stride_w,
                         int dil_h, int dil_w, int groups,
                         int n, int k, int p, int q)
{
    const int cg = C / groups;          /* input channels per group  */
    const int kg = K / groups;          /* filters per group         */
    const int c0 = (k / kg) * cg;       /* first input channel seen by filter k */
    double acc = 0.0;
    for (int c = 0; c < cg; ++c)
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s) {
                const int h  = p * stride_h - pad_h + r * dil_h;
                const int wv = q * stride_w - pad_w + s * dil_w;
                if (h < 0 || h >= H || wv < 0 || wv >= W) continue;   /* zero padding */
                const double xv = x[(((size_t)n * C + (c0 + c)) * H + h) * W + wv];
                const double fv = w[(((size_t)k * cg + c) * R + r) * S + s];
                acc += xv * fv;
            }
    return acc;
}

/*
 * Epilogue for one output: bias, optional inference batch-norm (per output channel), activation.
 * bn == NULL: no normalisation.  Otherwise bn points at 4 arrays of K doubles laid out
 * back to back: scale(gamma), shift(beta), mean, variance; eps is added to the variance.
 */
static double epilogue(double acc, const double *b, const double *bn, double eps,
                       int K, int k, int act, double alpha)
{
    double v = acc + (b ? b[k] : 0.0);
    if (bn) {
        const double gamma = bn[k], beta = bn[K + k], mean = bn[2 * K + k], var = bn[3 * K + k];
        v = gamma * (v - mean) / sqrt(var + eps) + beta;
    }
    return apply_act(v, act, alpha);
}

/*
 * Full forward pass.  x: N*C*H*W, w: K*(C/groups)*R*S, b: K or NULL, y: N*K*Ho*Wo (all packed,
 * row-major in the index order written).  Returns 0, or -1 on parameters that define no output.
 */
int conv_oracle_fwd(const double *x, const double *w, const double *b, const double *bn,
                    double eps, double *y,
                    int N, int C, int H, int W, int K, int R, int S,
                    int pad_h, int pad_w, int stride_h, int stride_w,
                    int dil_h, int dil_w, int groups, int act, double alpha)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1) return -1;
    if (pad_h < 0 || pad_w < 0 || stride_h < 1 || stride_w < 1 || dil_h < 1 || dil_w < 1) return -1;
    if (groups < 1 || C % groups || K % groups) return -1;
    const int Ho = conv_oracle_out_extent(H, R, pad_h, stride_h, dil_h);
    const int Wo = conv_oracle_out_extent(W, S, pad_w, stride_w, dil_w);
    if (Ho < 1 || Wo < 1) return -1;

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    const double acc = conv_point(x, w, C, H, W, K, R, S, pad_h, pad_w,
                                                  stride_h, stride_w, dil_h, dil_w, groups,
                                                  n, k, p, q);
                    y[(((size_t)n * K + k) * Ho + p) * Wo + q] =
                        epilogue(acc, b, bn, eps, K, k, act, alpha);
                }
    return 0;
}

/*
 * The same definition evaluated only at `count` chosen outputs: idx holds count quadruples
 * (n,k,p,q); out[i] receives y at the i-th quadruple.  Used to check full-size GPU results where
 * evaluating every output on the CPU would take too long.
 */
int conv_oracle_fwd_points(const double *x, const double *w, const double *b, const double *bn,
                           double eps, const int *idx, long count, double *out,
                           int N, int C, int H, int W, int K, int R, int S,
                           int pad_h, int pad_w, int stride_h, int stride_w,
                           int dil_h, int dil_w, int groups, int act, double alpha)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1) return -1;
    if (pad_h < 0 || pad_w < 0 || stride_h < 1 || stride_w < 1 || dil_h < 1 || dil_w < 1) return -1;
    if (groups < 1 || C % groups || K % groups) return -1;
    const int Ho = conv_oracle_out_extent(H, R, pad_h, stride_h, dil_h);
    const int Wo = conv_oracle_out_extent(W, S, pad_w, stride_w, dil_w);
    if (Ho < 1 || Wo < 1) return -1;
    for (long i = 0; i < count; ++i) {
        const int n = idx[4 * i], k = idx[4 * i + 1], p = idx[4 * i + 2], q = idx[4 * i + 3];
        if (n < 0 || n >= N || k < 0 || k >= K || p < 0 || p >= Ho || q < 0 || q >= Wo) return -2;
    }
#pragma omp parallel for schedule(static)
    for (long i = 0; i < count; ++i) {
        const int n = idx[4 * i], k = idx[4 * i + 1], p = idx[4 * i + 2], q = idx[4 * i + 3];
        const double acc = conv_point(x, w, C, H, W, K, R, S, pad_h, pad_w,
                                      stride_h, stride_w, dil_h, dil_w, groups, n, k, p, q);
        out[i] = epilogue(acc, b, bn, eps, K, k, act, alpha);
    }
    return 0;
}
