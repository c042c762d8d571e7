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
//   stem_wgrad_k   one workgroup per filter row (c, r), 8 output channels and
//                  chunk of output pixels, threads striding over the pixels;
//                  partial sums per chunk, added in a fixed order by
//                  stem_wgrad_reduce_k.
//   maxpool_fwd_k  one thread per output element.
//   maxpool_bwd_k  one thread per input element or per four of a row: it looks
//                  at the windows that contain them (winner codes written by
//                  maxpool_arg_k from the stored input) and takes the
//                  derivative of those they win.  A window's winner is its
//                  first maximal element in row-major order.  No atomics:
//                  results are reproducible.
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
// A workgroup owns 8 output channels and one filter row (c, r); its threads
// stride over the chunk's pixels, so the loads of dh (8 planes) and of the
// image row (KS neighbouring values) are coalesced across the lanes, and each
// thread keeps 8 x KS sums in registers.  At the end the sums are added over
// the workgroup: butterfly within a wavefront, then one thread per sum adds the
// four wavefronts' values in order.
template <int KS>
__global__ __launch_bounds__(kThreads) void stem_wgrad_k(const float *__restrict__ x, int64_t xsn, int64_t xsc,
                                                         const float *__restrict__ dh, int64_t dsn, int64_t dsc,
                                                         float *__restrict__ part, StemShape g, int64_t pixels,
                                                         int64_t per) {
    __shared__ float red[kThreads / 64][kWgradKG * KS];
    const int pad = (KS - 1) / 2, taps = g.CI * KS * KS;
    const int k0 = blockIdx.y * kWgradKG;
    const int c = blockIdx.z / KS, r = blockIdx.z - c * KS;
    const int HWO = g.HO * g.WO;
    float acc[kWgradKG][KS];
#pragma unroll
    for (int kk = 0; kk < kWgradKG; ++kk)
#pragma unroll
        for (int s = 0; s < KS; ++s) acc[kk][s] = 0.f;
    const int64_t i0 = (int64_t)blockIdx.x * per, i1 = min(pixels, i0 + per);
    for (int64_t i = i0 + threadIdx.x; i < i1; i += kThreads) {
        const int64_t n = i / HWO;
        const int pq = (int)(i - n * HWO);
        const int p = pq / g.WO, q = pq - p * g.WO;
        const int ih = p * g.stride + r - pad;
        if (ih < 0 || ih >= g.H) continue;
        const float *xrow = x + n * xsn + (int64_t)c * xsc + ih * g.W;
        float v[KS], d[kWgradKG];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int iw = q * g.stride + s - pad;
            v[s] = iw >= 0 && iw < g.W ? xrow[iw] : 0.f;
        }
        const float *dp = dh + n * dsn + pq;
#pragma unroll
        for (int kk = 0; kk < kWgradKG; ++kk) d[kk] = dp[(int64_t)min(k0 + kk, g.CO - 1) * dsc];
#pragma unroll
        for (int kk = 0; kk < kWgradKG; ++kk)
#pragma unroll
            for (int s = 0; s < KS; ++s) acc[kk][s] = fmaf(d[kk], v[s], acc[kk][s]);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int kk = 0; kk < kWgradKG; ++kk)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            float a = acc[kk][s];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
            if (lane == 0) red[wave][kk * KS + s] = a;
        }
    __syncthreads();
    if (threadIdx.x < kWgradKG * KS) {
        const int kk = threadIdx.x / KS, s = threadIdx.x - kk * KS;
        const float sum = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
        if (k0 + kk < g.CO)
            part[((int64_t)blockIdx.x * g.CO + (k0 + kk)) * taps + (c * KS + r) * KS + s] = sum;
    }
}

__global__ __launch_bounds__(kThreads) void stem_wgrad_reduce_k(const float *__restrict__ part, float *__restrict__ dw,
                                                                int chunks, int slots, int accumulate) {
    // 64 sums per workgroup; wavefront s adds the s-th quarter of the chunks in order (four loads in
    // flight), then the four quarters are added in a fixed order.
    __shared__ float red[kThreads / 64][64];
    const int lane = threadIdx.x & 63, share = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + lane, ic = min(i, slots - 1);
    const int per = (chunks + 3) / 4, c0 = share * per, c1 = min(chunks, c0 + per);
    float sum = 0.f;
    for (int c = c0; c < c1; c += 4) {
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = part[(int64_t)min(c + u, c1 - 1) * slots + ic];
#pragma unroll
        for (int u = 0; u < 4; ++u) sum += c + u < c1 ? v[u] : 0.f;
    }
    red[share][lane] = sum;
    __syncthreads();
    if (share == 0 && i < slots) {
        const float total = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
        dw[i] = accumulate ? dw[i] + total : total;
    }
}

// The first maximal element of window (p, q) in row-major order: its value and
// its position in the window, 3 * r + s.  All nine elements are requested
// before the first comparison (positions outside the plane re-read a valid one
// and are skipped), so the loads are in flight together.
__device__ __forceinline__ void window_winner(const float *plane, int H, int W, int p, int q, float *best, int *code) {
    float v[9];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int i = min(max(2 * p + r - 1, 0), H - 1);
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int j = min(max(2 * q + s - 1, 0), W - 1);
            v[3 * r + s] = plane[i * W + j];
        }
    }
    float b = -INFINITY;
    int w = 4;  // the centre is always inside the plane
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int i = 2 * p + r - 1;
#pragma unroll
        for (int s = 0; s < 3; ++s) {
            const int j = 2 * q + s - 1;
            const bool take = i >= 0 && i < H && j >= 0 && j < W && v[3 * r + s] > b;
            b = take ? v[3 * r + s] : b;
            w = take ? 3 * r + s : w;
        }
    }
    *best = b;
    *code = w;
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
    int code;
    window_winner(x + n * xsn + (int64_t)c * xsc, H, W, p, q, &best, &code);
    y[n * ysn + (int64_t)c * ysc + p * WO + q] = best;
}

// arg[n][c][p][q] = 3*r + s of the window's winner (dense bytes).
__global__ __launch_bounds__(kThreads) void maxpool_arg_k(const float *__restrict__ x, int64_t xsn, int64_t xsc,
                                                          unsigned char *__restrict__ arg, int C, int H, int W, int HO,
                                                          int WO, int64_t total) {
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= total) return;
    const int q = (int)(e % WO);
    int64_t t = e / WO;
    const int p = (int)(t % HO);
    t /= HO;
    const int c = (int)(t % C);
    const int64_t n = t / C;
    float best;
    int code;
    window_winner(x + n * xsn + (int64_t)c * xsc, H, W, p, q, &best, &code);
    arg[e] = (unsigned char)code;
}

// dx[n][c][i][j] (dense) = sum of dy over the windows that (i, j) wins, in a
// fixed order (window rows, then window columns).  A thread owns VEC
// consecutive j of one row (VEC = 4 needs W % 4 == 0; then the quad starts at
// an even j and lies in the windows q = j/2, j/2 + 1, j/2 + 2).  The winner
// codes and derivatives of those windows are requested up front, clamped to
// valid windows, and the ones that do not apply are masked.
template <int VEC>
__global__ __launch_bounds__(kThreads) void maxpool_bwd_k(const unsigned char *__restrict__ arg,
                                                          const float *__restrict__ dy, int64_t dsn, int64_t dsc,
                                                          float *__restrict__ dx, int C, int H, int W, int HO, int WO,
                                                          int64_t total) {
    constexpr int NQ = VEC == 4 ? 3 : 2;  // window columns a thread looks at
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // index of the thread's first element / VEC
    if (e >= total) return;
    const int wv = W / VEC;
    const int j0 = (int)(e % wv) * VEC;
    int64_t t = e / wv;
    const int i = (int)(t % H);
    t /= H;
    const int c = (int)(t % C);
    const int64_t n = t / C;
    const unsigned char *a = arg + (n * C + c) * (int64_t)(HO * WO);
    const float *g = dy + n * dsn + (int64_t)c * dsc;
    // window rows p with 2p-1 <= i <= 2p+1: i/2 and, for odd i, (i+1)/2
    const int p0 = i / 2, q0 = j0 / 2;
    int code[2][NQ];
    float d[2][NQ];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int p = min(p0 + u, HO - 1);
#pragma unroll
        for (int k = 0; k < NQ; ++k) {
            const int q = min(q0 + k, WO - 1);
            code[u][k] = a[p * WO + q];
            d[u][k] = g[p * WO + q];
        }
    }
    float out[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) out[k] = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int p = p0 + u;
        const bool row_ok = p < HO && (u == 0 || (i & 1));
#pragma unroll
        for (int k = 0; k < NQ; ++k) {
            const int q = q0 + k;
            // the winner's position in the plane
            const int wi = 2 * p - 1 + code[u][k] / 3, wj = 2 * q - 1 + code[u][k] % 3;
            const bool ok = row_ok && q < WO && wi == i;
#pragma unroll
            for (int m = 0; m < VEC; ++m) out[m] += ok && wj == j0 + m ? d[u][k] : 0.f;
        }
    }
    float *o = dx + ((n * C + c) * (int64_t)H + i) * W + j0;
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4 *>(o) = make_float4(out[0], out[1], out[2], out[3]);
    } else {
        o[0] = out[0];
    }
}

unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

}  // namespace

int stem_wgrad_chunks(const StemShape &g) {
    if (const int m = stem_wgrad_mfma_chunks(g)) return m;
    const int64_t pixels = (int64_t)g.N * g.HO * g.WO;
    const int64_t tiles = (int64_t)((g.CO + kWgradKG - 1) / kWgradKG) * g.CI * g.KS;  // workgroups per chunk
    int64_t chunks = (1024 + tiles - 1) / tiles;                 // about 1024 workgroups in all
    chunks = std::min<int64_t>(chunks, (pixels + 1023) / 1024);  // at least 1024 pixels each
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
    if (stem_conv_mfma_takes(g)) {
        stem_conv_mfma(cx, x, w, g, out);
        return;
    }
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
    if (stem_wgrad_mfma_chunks(g)) {
        if (cx.launch(K_STEM, 4.0 * ((double)g.N * g.CI * g.H * g.W + (double)pixels * g.CO), flops))
            stem_wgrad_mfma(cx, x, dh, g, scratch);
    } else if (cx.launch(K_STEM, 4.0 * ((double)g.N * g.CI * g.H * g.W + (double)pixels * g.CO), flops)) {
        const dim3 grid((unsigned)chunks, (unsigned)((g.CO + kWgradKG - 1) / kWgradKG), (unsigned)(g.CI * g.KS));
        const float *xp = x.p, *dp = dh.p;
        switch (g.KS) {
            case 1: cx.run(stem_wgrad_k<1>, grid, dim3(kThreads), 0, xp, x.sn, x.sc, dp, dh.sn, dh.sc, scratch, g, pixels, per); break;
            case 3: cx.run(stem_wgrad_k<3>, grid, dim3(kThreads), 0, xp, x.sn, x.sc, dp, dh.sn, dh.sc, scratch, g, pixels, per); break;
            case 5: cx.run(stem_wgrad_k<5>, grid, dim3(kThreads), 0, xp, x.sn, x.sc, dp, dh.sn, dh.sc, scratch, g, pixels, per); break;
            case 7: cx.run(stem_wgrad_k<7>, grid, dim3(kThreads), 0, xp, x.sn, x.sc, dp, dh.sn, dh.sc, scratch, g, pixels, per); break;
            default: cx.fail(hipErrorInvalidValue);  // larger kernels are refused by the caller
        }
    }
    if (cx.launch(K_STEM, 4.0 * (double)chunks * g.CO * taps))
        cx.run(stem_wgrad_reduce_k, dim3((unsigned)((g.CO * taps + 63) / 64)), dim3(kThreads), 0, (const float *)scratch, dw,
               chunks, g.CO * taps, accumulate ? 1 : 0);
}

void maxpool3s2_fwd(Ctx &cx, View x, int c, Geo in, View y) {
    const int ho = (in.h - 1) / 2 + 1, wo = (in.w - 1) / 2 + 1;
    const int64_t total = (int64_t)in.n * c * ho * wo;
    if (!cx.launch(K_STEM, 4.0 * ((double)in.pixels() * c + (double)total))) return;
    cx.run(maxpool_fwd_k, dim3(blocks_for(total)), dim3(kThreads), 0, (const float *)x.p, x.sn, x.sc, y.p, y.sn, y.sc, c, in.h,
           in.w, ho, wo, total);
}

size_t maxpool3s2_scratch_bytes(int c, Geo in) {
    return (size_t)in.n * c * ((in.h - 1) / 2 + 1) * ((in.w - 1) / 2 + 1);
}

void maxpool3s2_bwd(Ctx &cx, View x, View dy, int c, Geo in, unsigned char *scratch, float *dx) {
    const int ho = (in.h - 1) / 2 + 1, wo = (in.w - 1) / 2 + 1;
    const int64_t total = in.pixels() * c, outs = (int64_t)in.n * c * ho * wo;
    // the winners are found again from the stored input (one byte per window), then every input
    // element collects from the windows it won
    if (cx.launch(K_STEM, 4.0 * (double)total + (double)outs))
        cx.run(maxpool_arg_k, dim3(blocks_for(outs)), dim3(kThreads), 0, (const float *)x.p, x.sn, x.sc, scratch, c, in.h, in.w,
               ho, wo, outs);
    if (cx.launch(K_STEM, 4.0 * (double)total + 5.0 * (double)outs)) {
        // dx is dense; quads need rows of whole quads and a 16-byte aligned base
        if (in.w % 4 == 0 && (reinterpret_cast<uintptr_t>(dx) & 15) == 0)
            cx.run(maxpool_bwd_k<4>, dim3(blocks_for(total / 4)), dim3(kThreads), 0, (const unsigned char *)scratch,
                   (const float *)dy.p, dy.sn, dy.sc, dx, c, in.h, in.w, ho, wo, total / 4);
        else
            cx.run(maxpool_bwd_k<1>, dim3(blocks_for(total)), dim3(kThreads), 0, (const unsigned char *)scratch,
                   (const float *)dy.p, dy.sn, dy.sc, dx, c, in.h, in.w, ho, wo, total);
    }
}

}  // namespace rvn
