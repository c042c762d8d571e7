// Shape-generic direct convolutions (vector ALU, no matrix cores) for gfx950.
//
// These kernels accept every (c_in, c_out, k in {1,3}, h, w) the residual
// functions of Section 2.2 can ask for.  They are the path for shapes the
// matrix-core kernels do not cover.  Operands of a bf16 convolution are
// rounded to bf16 (nearest even) and multiplied in fp32, which is what a
// bf16 matrix instruction with fp32 accumulation computes up to summation
// order.
#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;
constexpr int kCoT = 8;      // output channels per thread
constexpr int kCiChunk = 32; // input channels staged per LDS round

__device__ __forceinline__ float bf16_round(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f;
    u += 0x7fffu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xffff0000u);
}

template <typename T>
__device__ __forceinline__ float load_elem(const T *p, int64_t i);
template <>
__device__ __forceinline__ float load_elem<float>(const float *p, int64_t i) {
    return p[i];
}
template <>
__device__ __forceinline__ float load_elem<uint16_t>(const uint16_t *p, int64_t i) {
    return __uint_as_float((uint32_t)p[i] << 16);
}

// out[n, o, p, q] = ep(r, sum_{i,r,s} in[n, i, p+r-pad, q+s-pad] * wt(o, i, r, s))
// with wt(o,i,r,s) = w[o][i][r][s]                       (forward,  TRANSPOSED = false)
//                  = w[i][o][KS-1-r][KS-1-s]             (data grad, TRANSPOSED = true)
// The data gradient of a stride-1 "same" convolution is itself such a
// convolution of the upstream gradient with the transposed, flipped filter.
template <int KS, typename TIN, bool TRANSPOSED>
__global__ __launch_bounds__(kThreads) void conv_direct_k(
    const TIN *__restrict__ in, int64_t isn, int64_t isc, int round_in, int round_w,
    const float *__restrict__ w, int CI, int CO, int N, int H, int W, int ep, const float *r,
    int64_t rsn, int64_t rsc, float *out, int64_t osn, int64_t osc) {
    __shared__ float wl[kCiChunk * KS * KS * kCoT];
    const int HW = H * W;
    const int64_t pix = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const bool live = pix < (int64_t)N * HW;
    const int n = live ? (int)(pix / HW) : 0;
    const int i_pl = live ? (int)(pix - (int64_t)n * HW) : 0;
    const int row = i_pl / W, col = i_pl - row * W;
    const int o0 = blockIdx.y * kCoT;
    constexpr int PAD = (KS - 1) / 2;

    float acc[kCoT];
#pragma unroll
    for (int j = 0; j < kCoT; ++j) acc[j] = 0.f;

    for (int c0 = 0; c0 < CI; c0 += kCiChunk) {
        const int cn = min(kCiChunk, CI - c0);
        __syncthreads();
        for (int e = threadIdx.x; e < cn * KS * KS * kCoT; e += kThreads) {
            const int j = e % kCoT;
            const int t = (e / kCoT) % (KS * KS);
            const int ci = e / (kCoT * KS * KS);
            const int o = o0 + j, i = c0 + ci;
            float v = 0.f;
            if (o < CO) {
                if (TRANSPOSED) {
                    const int rr = KS - 1 - t / KS, ss = KS - 1 - t % KS;
                    v = w[((int64_t)i * CO + o) * (KS * KS) + rr * KS + ss];
                } else {
                    v = w[((int64_t)o * CI + i) * (KS * KS) + t];
                }
                if (round_w) v = bf16_round(v);
            }
            wl[e] = v;
        }
        __syncthreads();
        if (live) {
            const TIN *src = in + (int64_t)n * isn + (int64_t)c0 * isc;
            for (int ci = 0; ci < cn; ++ci) {
#pragma unroll
                for (int rr = 0; rr < KS; ++rr) {
                    const int ih = row + rr - PAD;
#pragma unroll
                    for (int ss = 0; ss < KS; ++ss) {
                        const int iw = col + ss - PAD;
                        float v = 0.f;
                        if (ih >= 0 && ih < H && iw >= 0 && iw < W) {
                            v = load_elem<TIN>(src, (int64_t)ci * isc + ih * W + iw);
                            if (round_in) v = bf16_round(v);
                        }
                        const float *wp = &wl[(ci * KS * KS + rr * KS + ss) * kCoT];
#pragma unroll
                        for (int j = 0; j < kCoT; ++j) acc[j] = fmaf(v, wp[j], acc[j]);
                    }
                }
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int j = 0; j < kCoT; ++j) {
        const int o = o0 + j;
        if (o >= CO) break;
        float v = acc[j];
        if (ep != EP_STORE) {
            const float rv = r[(int64_t)n * rsn + (int64_t)o * rsc + i_pl];
            v = ep == EP_ADD ? rv + v : rv - v;
        }
        out[(int64_t)n * osn + (int64_t)o * osc + i_pl] = v;
    }
}

// Filter gradient, partial over an image group:
//   part[s][k][c][t] = sum_{n in group s} sum_{p,q} dh[n,k,p,q] * a[n,c,p+r-pad,q+s-pad]
// One workgroup per (k, group of kCT input channels, image group).
constexpr int kCT = 4;

template <int KS, typename TA>
__global__ __launch_bounds__(kThreads) void wgrad_direct_partial_k(
    const TA *__restrict__ a, const float *__restrict__ dh, int64_t dsn, int64_t dsc, int round_dh,
    int CI, int CO, int N, int H, int W, int ipw, float *__restrict__ part) {
    constexpr int T = KS * KS, PAD = (KS - 1) / 2;
    __shared__ float lds[4 * T * kCT];
    const int k = blockIdx.x, c0 = blockIdx.y * kCT, s = blockIdx.z;
    const int HW = H * W;
    const int n0 = s * ipw, n1 = min(N, n0 + ipw);
    float acc[T * kCT];
#pragma unroll
    for (int j = 0; j < T * kCT; ++j) acc[j] = 0.f;
    for (int n = n0; n < n1; ++n) {
        const float *pd = dh + (int64_t)n * dsn + (int64_t)k * dsc;
        const TA *pa = a + ((int64_t)n * CI + c0) * HW;
        for (int i = threadIdx.x; i < HW; i += kThreads) {
            float g = pd[i];
            if (round_dh) g = bf16_round(g);
            const int row = i / W, col = i - row * W;
#pragma unroll
            for (int cc = 0; cc < kCT; ++cc) {
                if (c0 + cc >= CI) break;
#pragma unroll
                for (int rr = 0; rr < KS; ++rr) {
                    const int ih = row + rr - PAD;
#pragma unroll
                    for (int ss = 0; ss < KS; ++ss) {
                        const int iw = col + ss - PAD;
                        float v = 0.f;
                        if (ih >= 0 && ih < H && iw >= 0 && iw < W)
                            v = load_elem<TA>(pa, (int64_t)cc * HW + ih * W + iw);
                        acc[cc * T + rr * KS + ss] = fmaf(g, v, acc[cc * T + rr * KS + ss]);
                    }
                }
            }
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int j = 0; j < T * kCT; ++j) {
        float v = acc[j];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
        if (lane == 0) lds[wave * T * kCT + j] = v;
    }
    __syncthreads();
    if (threadIdx.x < T * kCT) {
        const int j = threadIdx.x, cc = j / T, t = j % T;
        if (c0 + cc < CI) {
            const float v = (lds[j] + lds[T * kCT + j]) + (lds[2 * T * kCT + j] + lds[3 * T * kCT + j]);
            part[(((int64_t)s * CO + k) * CI + c0 + cc) * T + t] = v;
        }
    }
}

// dw[i] (+)= sum_s part[s][i], in order.
__global__ void reduce_partials_k(const float *__restrict__ part, int64_t count, int S,
                                  float *__restrict__ dw, int accumulate) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    float v = 0.f;
    for (int s = 0; s < S; ++s) v += part[(int64_t)s * count + i];
    dw[i] = accumulate ? dw[i] + v : v;
}

int wgrad_splits(int cin, int cout, const Geo &g) {
    const int64_t base = (int64_t)cout * ((cin + kCT - 1) / kCT);
    int64_t s = (2048 + base - 1) / base;
    if (s > g.n) s = g.n;
    if (s < 1) s = 1;
    const int ipw = (int)((g.n + s - 1) / s);
    return (g.n + ipw - 1) / ipw;
}

}  // namespace

size_t wgrad_scratch_floats(int cin, int cout, int ks, const Geo &g) {
    return (size_t)wgrad_splits(cin, cout, g) * cin * cout * ks * ks;
}

static void conv_common(Ctx &cx, const void *in, bool in_bf16_storage, int64_t isn, int64_t isc,
                        bool round_in, bool round_w, bool transposed, const float *w, int ci, int co,
                        int ks, Geo g, Epilogue ep, const View *r, View out) {
    dim3 grid((unsigned)((g.pixels() + kThreads - 1) / kThreads), (co + kCoT - 1) / kCoT);
    const float *rp = r ? r->p : nullptr;
    const int64_t rsn = r ? r->sn : 0, rsc = r ? r->sc : 0;
#define RVN_LAUNCH(KS, T, TR)                                                                      \
    conv_direct_k<KS, T, TR><<<grid, kThreads, 0, cx.stream>>>(                                    \
        static_cast<const T *>(in), isn, isc, round_in ? 1 : 0, round_w ? 1 : 0, w, ci, co, g.n, g.h, \
        g.w, (int)ep, rp, rsn, rsc, out.p, out.sn, out.sc)
    if (ks == 3) {
        if (transposed) RVN_LAUNCH(3, float, true);
        else if (in_bf16_storage) RVN_LAUNCH(3, uint16_t, false);
        else RVN_LAUNCH(3, float, false);
    } else {
        if (transposed) RVN_LAUNCH(1, float, true);
        else if (in_bf16_storage) RVN_LAUNCH(1, uint16_t, false);
        else RVN_LAUNCH(1, float, false);
    }
#undef RVN_LAUNCH
    cx.check();
}

void conv_fwd(Ctx &cx, const void *a, rvn_dtype dt, const float *w, int cin, int cout, int ks,
              Geo g, Epilogue ep, const View *r, View out) {
    const double P = (double)g.pixels();
    const double esz = dt == RVN_BF16 ? 2.0 : 4.0;
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_fwd_calls += 1;
    cx.cost.conv_flops += flops;
    if (!cx.launch(K_CONV_FWD, P * cin * esz + P * cout * 4.0 * (ep == EP_STORE ? 1.0 : 2.0), flops)) return;
    conv_common(cx, a, dt == RVN_BF16, (int64_t)cin * g.hw(), g.hw(), false, dt == RVN_BF16, false, w,
                cin, cout, ks, g, ep, r, out);
}

void conv_dgrad(Ctx &cx, View dh, rvn_dtype dt, const float *w, int cin, int cout, int ks, Geo g,
                float *da) {
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_dgrad_calls += 1;
    cx.cost.conv_flops += flops;
    if (!cx.launch(K_CONV_DGRAD, P * cout * 4.0 + P * cin * 4.0, flops)) return;
    // The "input" of this convolution is dh with `cout` channels; it produces `cin` channels.
    conv_common(cx, dh.p, false, dh.sn, dh.sc, dt == RVN_BF16, dt == RVN_BF16, true, w, cout, cin, ks, g,
                EP_STORE, nullptr, dense_view(da, cin, g));
}

void conv_wgrad(Ctx &cx, const void *a, rvn_dtype dt, View dh, int cin, int cout, int ks, Geo g,
                float *scratch, float *dw, bool accumulate) {
    const double P = (double)g.pixels();
    const double esz = dt == RVN_BF16 ? 2.0 : 4.0;
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_wgrad_calls += 1;
    cx.cost.conv_flops += flops;
    const int S = wgrad_splits(cin, cout, g);
    const int ipw = (g.n + S - 1) / S;
    if (cx.launch(K_CONV_WGRAD, P * cin * esz + P * cout * 4.0, flops)) {
        dim3 grid(cout, (cin + kCT - 1) / kCT, S);
#define RVN_LAUNCH(KS, T)                                                                   \
    wgrad_direct_partial_k<KS, T><<<grid, kThreads, 0, cx.stream>>>(                        \
        static_cast<const T *>(a), dh.p, dh.sn, dh.sc, dt == RVN_BF16 ? 1 : 0, cin, cout, g.n, g.h, \
        g.w, ipw, scratch)
        if (ks == 3) {
            if (dt == RVN_BF16) RVN_LAUNCH(3, uint16_t);
            else RVN_LAUNCH(3, float);
        } else {
            if (dt == RVN_BF16) RVN_LAUNCH(1, uint16_t);
            else RVN_LAUNCH(1, float);
        }
#undef RVN_LAUNCH
        cx.check();
    }
    if (cx.launch(K_WGRAD_REDUCE, 0.0)) {
        const int64_t count = (int64_t)cin * cout * ks * ks;
        reduce_partials_k<<<(unsigned)((count + 255) / 256), 256, 0, cx.stream>>>(scratch, count, S, dw, accumulate ? 1 : 0);
        cx.check();
    }
}

}  // namespace rvn
