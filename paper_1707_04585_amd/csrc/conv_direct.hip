// Shape-generic filter gradient on the vector ALU (no matrix cores) for gfx950.
//
// Accepts every (c_in, c_out, k in {1,3}, h, w) the residual functions of
// Section 2.2 can ask for.  Operands of a bf16 convolution are rounded to bf16
// (nearest even) and multiplied in fp32, which is what a bf16 matrix
// instruction with fp32 accumulation computes up to summation order.
#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;

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
