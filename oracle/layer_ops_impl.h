/*
 * TEST INFRASTRUCTURE ONLY -- CPU oracle for the reversible-residual-network
 * hot path.  Nothing in the product (the HIP library, its Python binding) may
 * include, link or call this file; only tests, the smoke check and the
 * benchmark's cpu_baseline leg do.
 *
 * This header is included twice by layer_ops.c, once with REAL=double
 * (suffix _f64) and once with REAL=float (suffix _f32).  It holds the layer
 * level definitions the paper relies on (Section 2.2, the equation defining
 * a(x), c_k(x), Basic and Bottleneck):
 *
 *   a(x)   = ReLU(BN(x))            train-mode batch normalisation, then ReLU
 *   c_k(x) = Conv_{k x k}(a(x))     k in {1,3}
 *
 * and their reverse-mode derivatives, each written as the plain definition
 * (Section 2.1, the backprop rule: the adjoint of a node is the sum over its
 * children of Jacobian-transpose times the child's adjoint).  There is no
 * blocking, fusion or reordering: every routine is a direct loop nest over the
 * mathematical index set.
 *
 * Layout: dense NCHW, row major.  Filters: [K][C][k][k].  Zero padding
 * (k-1)/2, dilation 1, one group, no bias, cross-correlation (no filter
 * flip).  `stride` is 1 inside reversible blocks (Section 3.1: a reversible
 * block must have stride 1); other strides exist only for the non-reversible
 * subsampling layers between stages.
 */

/* out[n,k,p,q] = sum_{c,r,s} a[n,c,p*stride+r-pad,q*stride+s-pad] * w[k,c,r,s] */
void FN(orc_conv_fwd)(const REAL *a, const REAL *w, REAL *out,
                      int N, int C, int K, int H, int W, int ks, int stride)
{
    const int pad = (ks - 1) / 2;
    const int Ho = (H + 2 * pad - ks) / stride + 1;
    const int Wo = (W + 2 * pad - ks) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    REAL acc = 0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < ks; ++r)
                            for (int s = 0; s < ks; ++s) {
                                const int ih = p * stride + r - pad;
                                const int iw = q * stride + s - pad;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W)
                                    continue;
                                acc += a[(((size_t)n * C + c) * H + ih) * W + iw] *
                                       w[(((size_t)k * C + c) * ks + r) * ks + s];
                            }
                    out[(((size_t)n * K + k) * Ho + p) * Wo + q] = acc;
                }
}

/* Adjoint with respect to the input: every forward product a*w contributes
 * dout*w to da at the input position it read.  Written as the transpose of
 * the forward loop nest (a scatter), not as a second convolution. */
void FN(orc_conv_dgrad)(const REAL *dout, const REAL *w, REAL *da,
                        int N, int C, int K, int H, int W, int ks, int stride)
{
    const int pad = (ks - 1) / 2;
    const int Ho = (H + 2 * pad - ks) / stride + 1;
    const int Wo = (W + 2 * pad - ks) / stride + 1;
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        REAL *dan = da + (size_t)n * C * H * W;
        for (size_t i = 0; i < (size_t)C * H * W; ++i)
            dan[i] = 0;
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    const REAL g = dout[(((size_t)n * K + k) * Ho + p) * Wo + q];
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < ks; ++r)
                            for (int s = 0; s < ks; ++s) {
                                const int ih = p * stride + r - pad;
                                const int iw = q * stride + s - pad;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W)
                                    continue;
                                dan[((size_t)c * H + ih) * W + iw] +=
                                    g * w[(((size_t)k * C + c) * ks + r) * ks + s];
                            }
                }
    }
}

/* Adjoint with respect to the filter: dw[k,c,r,s] = sum over every forward
 * product that used w[k,c,r,s] of dout times the input value it multiplied. */
void FN(orc_conv_wgrad)(const REAL *a, const REAL *dout, REAL *dw,
                        int N, int C, int K, int H, int W, int ks, int stride)
{
    const int pad = (ks - 1) / 2;
    const int Ho = (H + 2 * pad - ks) / stride + 1;
    const int Wo = (W + 2 * pad - ks) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < ks; ++r)
                for (int s = 0; s < ks; ++s) {
                    REAL acc = 0;
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < Ho; ++p) {
                            const int ih = p * stride + r - pad;
                            if (ih < 0 || ih >= H)
                                continue;
                            for (int q = 0; q < Wo; ++q) {
                                const int iw = q * stride + s - pad;
                                if (iw < 0 || iw >= W)
                                    continue;
                                acc += dout[(((size_t)n * K + k) * Ho + p) * Wo + q] *
                                       a[(((size_t)n * C + c) * H + ih) * W + iw];
                            }
                        }
                    dw[(((size_t)k * C + c) * ks + r) * ks + s] = acc;
                }
}

/* a(x) = ReLU(BN(x)), train mode.  Two-pass statistics over the M = N*H*W
 * values of each channel: mean first, then the biased variance of the
 * centred values.  Stores what the stored-activation backward pass needs:
 * xhat (normalised), u (affine output before the ReLU), a (after it). */
void FN(orc_bn_relu_fwd)(const REAL *x, const REAL *gamma, const REAL *beta, REAL eps,
                         REAL *mean, REAL *var, REAL *xhat, REAL *u, REAL *a,
                         int N, int C, int H, int W)
{
    const size_t HW = (size_t)H * W;
    const REAL M = (REAL)((size_t)N * HW);
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        REAL s = 0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i)
                s += x[((size_t)n * C + c) * HW + i];
        const REAL mu = s / M;
        REAL v = 0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const REAL d = x[((size_t)n * C + c) * HW + i] - mu;
                v += d * d;
            }
        v /= M;
        mean[c] = mu;
        var[c] = v;
        const REAL sd = (REAL)sqrt((double)(v + eps));
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const size_t j = ((size_t)n * C + c) * HW + i;
                const REAL xh = (x[j] - mu) / sd;
                const REAL uu = gamma[c] * xh + beta[c];
                xhat[j] = xh;
                u[j] = uu;
                a[j] = uu > 0 ? uu : 0;
            }
    }
}

/* Reverse mode through a = ReLU(u), u = gamma*xhat + beta,
 * xhat = (x - mu)/sqrt(var + eps), var = mean((x-mu)^2), mu = mean(x),
 * one graph node at a time (the unfused chain rule; the derivative of the
 * ReLU at 0 is taken as 0). */
void FN(orc_bn_relu_bwd)(const REAL *da, const REAL *x, const REAL *gamma, REAL eps,
                         const REAL *mean, const REAL *var, const REAL *xhat, const REAL *u,
                         REAL *dx, REAL *dgamma, REAL *dbeta,
                         int N, int C, int H, int W)
{
    const size_t HW = (size_t)H * W;
    const REAL M = (REAL)((size_t)N * HW);
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        const REAL mu = mean[c];
        const REAL ve = var[c] + eps;
        const REAL sd = (REAL)sqrt((double)ve);
        REAL dg = 0, db = 0, dvar = 0, dmu_direct = 0, sum_centred = 0;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const size_t j = ((size_t)n * C + c) * HW + i;
                const REAL du = u[j] > 0 ? da[j] : 0;      /* ReLU node   */
                dg += du * xhat[j];                        /* u = g*xh+b  */
                db += du;
                const REAL dxh = du * gamma[c];
                /* xhat = (x-mu) * (var+eps)^(-1/2) */
                dvar += dxh * (x[j] - mu) * ((REAL)-0.5) / (ve * sd);
                dmu_direct += -dxh / sd;
                sum_centred += x[j] - mu;
            }
        /* var = mean((x-mu)^2) also depends on mu */
        const REAL dmu = dmu_direct + dvar * ((REAL)-2) * sum_centred / M;
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const size_t j = ((size_t)n * C + c) * HW + i;
                const REAL du = u[j] > 0 ? da[j] : 0;
                const REAL dxh = du * gamma[c];
                dx[j] = dxh / sd + dvar * 2 * (x[j] - mu) / M + dmu / M;
            }
        dgamma[c] = dg;
        dbeta[c] = db;
    }
}
