// The network's first layers, ahead of the reversible stages (Section 3.2:
// non-reversible layers, whose inputs are stored): a k x k convolution of the
// image with stride 1 or 2, and 3x3 stride-2 max-pooling.  The image has a
// handful of channels, so the reduction is far too short for the matrix cores'
// implicit-GEMM kernels (c_in * k * k = 27 or 147 against tiles of 16 input
// channels per tap); these are direct kernels on the vector ALUs, fp32.
//
//   stem_conv_k    one thread per output pixel and 16 output channels; the
//                  filters of those channels sit in LDS and are read as
//                  broadcasts, the image through the vector cache.
//   stem_wgrad_k   one thread per filter tap (c, r, s) and 8 output channels,
//                  one workgroup per chunk of output pixels; partial sums per
//                  chunk, added in a fixed order by stem_wgrad_reduce_k.
//   maxpool_fwd_k  one thread per output element.
//   maxpool_bwd_k  one thread per input element: it looks at the (at most four)
//                  windows that contain it and takes the derivative of those
//                  it wins.  A window's winner is its first maximal element in
//                  row-major order.  No atomics: results are reproducible.
#include <algorithm>

#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;
constexpr int kConvKG = 16;   // output channels per thread, forward
constexpr int kWgradKG = 8;   // output channels per thread, filter gradient

__global__ __launch_bounds__(kThreads) void stem_conv_k(const float *__restrict__ x, int64_t xsn, int64_t xsc,
                                                        const float *__restrict__ w, float *__restrict__ out,
                                                        int64_t osn, int64_t osc, StemShape g, int64_t pixels) {
    extern __shared__ float wl[];  // [taps][kConvKG]
    const int taps = g.CI * g.KS * g.KS, pad = (g.KS - 1) / 2;
    const int k0 = blockIdx.y * kConvKG;
    for (int e = threadIdx.x; e < taps * kConvKG; e += kThreads) {
        const int t = e / kConvKG, kk = e - t * kConvKG;
        wl[e] = k0 + kk < g.CO ? w[(int64_t)(k0 + kk) * taps + t] : 0.f;
    }
    __syncthreads();
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= pixels) return;
    const int q = (int)(i % g.WO);
    const int64_t t1 = i / g.WO;
    const int p = (int)(t1 % g.HO);
    const int64_t n = t1 / g.HO;
    float acc[kConvKG];
#pragma unroll
    for (int kk = 0; kk < kConvKG; ++kk) acc[kk] = 0.f;
    const float *xn = x + n * xsn;
    int tap = 0;
    for (int c = 0; c < g.CI; ++c)
        for (int r = 0; r < g.KS; ++r) {
            const int ih = p * g.stride + r - pad;
            for (int s = 0; s < g.KS; ++s, ++tap) {
                const int iw = q * g.stride + s - pad;
                const bool in = ih >= 0 && ih < g.H && iw >= 0 && iw < g.W;
                const float v = in ? xn[(int64_t)c * xsc + ih * g.W + iw] : 0.f;
                const float *wt = wl + tap * kConvKG;
#pragma unroll
                for (int kk = 0; kk < kConvKG; ++kk) acc[kk] = fmaf(v, wt[kk], acc[kk]);
            }
        }
    float *on = out + n * osn + p * g.WO + q;
#pragma unroll
    for (int kk = 0; kk < kConvKG; ++kk)
        if (k0 + kk < g.CO) on[(int64_t)(k0 + kk) * osc] = acc[kk];
}

// part[chunk][k][tap] over the chunk's output pixels [chunk*per, (chunk+1)*per).
__global__ __launch_bounds__(kThreads) void stem_wgrad_k(const float *__restrict__ x, int64_t xsn, int64_t xsc,
                                                         const float *__restrict__ dh, int64_t dsn, int64_t dsc,
                                                         float *__restrict__ part, StemShape g, int64_t pixels,
                                                         int64_t per) {
    const int taps = g.CI * g.KS * g.KS, pad = (g.KS - 1) / 2;
    const int t = threadIdx.x;
    if (t >= taps) return;
    const int c = t / (g.KS * g.KS), rs = t - c * (g.KS * g.KS), r = rs / g.KS, s = rs - r * g.KS;
    const int k0 = blockIdx.y * kWgradKG;
    float acc[kWgradKG];
#pragma unroll
    for (int kk = 0; kk < kWgradKG; ++kk) acc[kk] = 0.f;
    const int64_t i0 = (int64_t)blockIdx.x * per, i1 = min(pixels, i0 + per);
    int q = (int)(i0 % g.WO);
    int64_t t1 = i0 / g.WO;
    int p = (int)(t1 % g.HO);
    int64_t n = t1 / g.HO;
    for (int64_t i = i0; i < i1; ++i) {
        const int ih = p * g.stride + r - pad, iw = q * g.stride + s - pad;
        const bool in = ih >= 0 && ih < g.H && iw >= 0 && iw < g.W;
        const float v = in ? x[n * xsn + (int64_t)c * xsc + ih * g.W + iw] : 0.f;
        const float *d = dh + n * dsn + p * g.WO + q;  // the same address in every lane: one request
#pragma unroll
        for (int kk = 0; kk < kWgradKG; ++kk) {
            const int k = min(k0 + kk, g.CO - 1);
            acc[kk] = fmaf(d[(int64_t)k * dsc], v, acc[kk]);
        }
        if (++q == g.WO) {
            q = 0;
            if (++p == g.HO) {
                p = 0;
                ++n;
            }
        }
    }
    float *o = part + ((int64_t)blockIdx.x * g.CO) * taps;
#pragma unroll
    for (int kk = 0; kk < kWgradKG; ++kk)
        if (k0 + kk < g.CO) o[(int64_t)(k0 + kk) * taps + t] = acc[kk];
}

__global__ __launch_bounds__(kThreads) void stem_wgrad_reduce_k(const float *__restrict__ part, float *__restrict__ dw,
                                                                int chunks, int slots, int accumulate) {
    const int i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= slots) return;
    float sum = 0.f;
    for (int s = 0; s < chunks; ++s) sum += part[(int64_t)s * slots + i];
    dw[i] = accumulate ? dw[i] + sum : sum;
}

// The first maximal element of window (p, q) in row-major order; returns its value and position.
__device__ __forceinline__ void window_winner(const float *plane, int H, int W, int p, int q, float *best, int *bi, int *bj) {
    float b = -INFINITY;
    int wi = -1, wj = -1;
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int i = 2 * p + r - 1;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int j = 2 * q + s - 1;
            if (i < 0 || i >= H || j < 0 || j >= W) continue;
            const float v = plane[i * W + j];
            if (v > b) {
                b = v;
                wi = i;
                wj = j;
            }
        }
    }
    *best = b;
    *bi = wi;
    *bj = wj;
}

__global__ __launch_bounds__(kThreads) void maxpool_fwd_k(const float *__restrict__ x, int64_t xsn, int64_t xsc,
                                                          float *__restrict__ y, int64_t ysn, int64_t ysc, int C, int H,
                                                          int W, int HO, int WO, int64_t total) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= total) return;
    const int q = (int)(e % WO);
    int64_t t = e / WO;
    const int p = (int)(t % HO);
    t /= HO;
    const int c = (int)(t % C);
    const int64_t n = t / C;
    float best;
    int bi, bj;
    window_winner(x + n * xsn + (int64_t)c * xsc, H, W, p, q, &best, &bi, &bj);
    y[n * ysn + (int64_t)c * ysc + p * WO + q] = best;
}

__global__ __launch_bounds__(kThreads) void maxpool_bwd_k(const float *__restrict__ x, int64_t xsn, int64_t xsc,
                                                          const float *__restrict__ dy, int64_t dsn, int64_t dsc,
                                                          float *__restrict__ dx, int C, int H, int W, int HO, int WO,
                                                          int64_t total) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= total) return;
    const int j = (int)(e % W);
    int64_t t = e / W;
    const int i = (int)(t % H);
    t /= H;
    const int c = (int)(t % C);
    const int64_t n = t / C;
    const float *plane = x + n * xsn + (int64_t)c * xsc;
    const float *g = dy + n * dsn + (int64_t)c * dsc;
    // windows p with 2p-1 <= i <= 2p+1
    const int p_lo = max(0, i / 2), p_hi = min(HO - 1, (i + 1) / 2);
    const int q_lo = max(0, j / 2), q_hi = min(WO - 1, (j + 1) / 2);
    float sum = 0.f;
    for (int p = p_lo; p <= p_hi; ++p)
        for (int q = q_lo; q <= q_hi; ++q) {
            float best;
            int bi, bj;
            window_winner(plane, H, W, p, q, &best, &bi, &bj);
            if (bi == i && bj == j) sum += g[p * WO + q];
        }
    dx[e] = sum;  // dense [n][c][h][w]
}

unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

}  // namespace

int stem_wgrad_chunks(const StemShape &g) {
    const int64_t pixels = (int64_t)g.N * g.HO * g.WO;
    const int groups = (g.CO + kWgradKG - 1) / kWgradKG;
    int64_t chunks = std::max<int64_t>(1, 2048 / groups);
    chunks = std::min<int64_t>(chunks, (pixels + 255) / 256);  // at least 256 pixels each
    return (int)std::max<int64_t>(chunks, 1);
}

size_t stem_wgrad_scratch_floats(const StemShape &g) {
    return (size_t)stem_wgrad_chunks(g) * g.CO * g.CI * g.KS * g.KS;
}

void stem_conv(Ctx &cx, View x, const float *w, const StemShape &g, View out) {
    const int64_t pixels = (int64_t)g.N * g.HO * g.WO;
    const int taps = g.CI * g.KS * g.KS;
    const double flops = 2.0 * (double)pixels * g.CO * taps;
    cx.cost.conv_fwd_calls += 1;
    cx.cost.conv_flops += flops;
    if (!cx.launch(K_STEM, 4.0 * ((double)g.N * g.CI * g.H * g.W + (double)pixels * g.CO), flops)) return;
    const dim3 grid(blocks_for(pixels), (unsigned)((g.CO + kConvKG - 1) / kConvKG));
    cx.run(stem_conv_k, grid, dim3(kThreads), (size_t)taps * kConvKG * 4, (const float *)x.p, x.sn, x.sc, w, out.p, out.sn,
           out.sc, g, pixels);
}

void stem_wgrad(Ctx &cx, View x, View dh, const StemShape &g, float *scratch, float *dw, bool accumulate) {
    const int64_t pixels = (int64_t)g.N * g.HO * g.WO;
    const int taps = g.CI * g.KS * g.KS;
    const double flops = 2.0 * (double)pixels * g.CO * taps;
    cx.cost.conv_wgrad_calls += 1;
    cx.cost.conv_flops += flops;
    const int chunks = stem_wgrad_chunks(g);
    const int64_t per = (pixels + chunks - 1) / chunks;
    if (cx.launch(K_STEM, 4.0 * ((double)g.N * g.CI * g.H * g.W + (double)pixels * g.CO), flops)) {
        const dim3 grid((unsigned)chunks, (unsigned)((g.CO + kWgradKG - 1) / kWgradKG));
        cx.run(stem_wgrad_k, grid, dim3(kThreads), 0, (const float *)x.p, x.sn, x.sc, (const float *)dh.p, dh.sn, dh.sc,
               scratch, g, pixels, per);
    }
    if (cx.launch(K_STEM, 4.0 * (double)chunks * g.CO * taps))
        cx.run(stem_wgrad_reduce_k, dim3(blocks_for((int64_t)g.CO * taps)), dim3(kThreads), 0, (const float *)scratch, dw,
               chunks, g.CO * taps, accumulate ? 1 : 0);
}

void maxpool3s2_fwd(Ctx &cx, View x, int c, Geo in, View y) {
    const int ho = (in.h - 1) / 2 + 1, wo = (in.w - 1) / 2 + 1;
    const int64_t total = (int64_t)in.n * c * ho * wo;
    if (!cx.launch(K_STEM, 4.0 * ((double)in.pixels() * c + (double)total))) return;
    cx.run(maxpool_fwd_k, dim3(blocks_for(total)), dim3(kThreads), 0, (const float *)x.p, x.sn, x.sc, y.p, y.sn, y.sc, c, in.h,
           in.w, ho, wo, total);
}

void maxpool3s2_bwd(Ctx &cx, View x, View dy, int c, Geo in, float *dx) {
    const int ho = (in.h - 1) / 2 + 1, wo = (in.w - 1) / 2 + 1;
    const int64_t total = in.pixels() * c;
    if (!cx.launch(K_STEM, 4.0 * (2.0 * (double)total + (double)in.n * c * ho * wo))) return;
    cx.run(maxpool_bwd_k, dim3(blocks_for(total)), dim3(kThreads), 0, (const float *)x.p, x.sn, x.sc, (const float *)dy.p,
           dy.sn, dy.sc, dx, c, in.h, in.w, ho, wo, total);
}

}  // namespace rvn
