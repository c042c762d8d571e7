// Data gradient and filter gradient of one fp32 layer in a single launch.
//
// Both need only the upstream gradient dh (Algorithm 1: the "ordinary backprop"
// steps), so they are independent; at the sizes of the CIFAR-like stacks each
// is bound by per-launch latency rather than by a pipe.  One launch holds the
// workgroups of both (filter gradient first: it has the longer dependent chain),
// which saves a launch and lets the matrix phases of one overlap the load and
// store phases of the other on the same compute units.
#include <cstdlib>

#include "conv_mfma_body.h"
#include "conv_wgrad_body.h"
#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;

template <int KS, int CMT, int CNT, int CKC, int WMT, int WCT>
__global__ __launch_bounds__(kThreads) void dgrad_wgrad_f32_k(const ConvArgs c, const WgradArgs w, int w_gx, int w_gy,
                                                              int w_gz, int c_gx) {
    extern __shared__ __align__(16) float smem[];
    const int n_w = w_gx * w_gy * w_gz;
    if ((int)blockIdx.x < n_w) {
        const int bx = blockIdx.x % w_gx, t = blockIdx.x / w_gx;
        conv_wgrad_mfma_body<KS, WMT, WCT, true>(w, bx, t % w_gy, t / w_gy, w_gz, smem);
    } else {
        const int b = blockIdx.x - n_w;
        conv_mfma_f32_body<KS, CMT, CNT, CKC>(c, b % c_gx, b / c_gx, smem);
    }
}

}  // namespace

bool separate_launches() {
    const char *e = std::getenv("RVN_SEPARATE_LAUNCHES");
    return e && e[0] == '1' && e[1] == 0;
}

bool conv_dgrad_wgrad_f32(Ctx &cx, View x, const float *scale_shift, View dh, const float *w, int cin, int cout,
                          int ks, Geo g, float *scratch, float *dw, bool accumulate, float *da, WgradReduce *defer) {
    if (ks != 3 || !defer || separate_launches()) return false;
    ConvLaunch C;
    WgradLaunch W;
    WgradReduce red{};
    // data gradient: a stride-1 "same" convolution of dh (cout channels) with the
    // transposed, flipped filter, producing cin channels
    if (!conv_mfma_plan(dh, nullptr, w, true, cout, cin, ks, g, false, EP_STORE, nullptr, dense_view(da, cin, g), C)) return false;
    if (!conv_wgrad_plan(x, scale_shift, false, dh, cin, cout, ks, g, scratch, dw, accumulate, W, red)) return false;
    if (!W.vec || C.nt != 4 || C.kc != 16) return false;
    const bool small = C.mt == 1 && W.mt == 1 && W.ct == 1, mid = C.mt == 2 && W.mt == 2 && W.ct == 2;
    if (!small && !mid) return false;
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_dgrad_calls += 1;
    cx.cost.conv_wgrad_calls += 1;
    cx.cost.conv_flops += 2.0 * flops;
    *defer = red;
    if (!cx.launch(K_CONV_DGRAD_WGRAD, 2.0 * (P * cin * 4.0 + P * cout * 4.0), 2.0 * flops)) return true;
    const unsigned n_w = W.grid.x * W.grid.y * W.grid.z, n_c = C.grid.x * C.grid.y;
    const size_t lds = std::max(C.lds_bytes, W.lds_bytes);
    if (small)
        cx.run(dgrad_wgrad_f32_k<3, 1, 4, 16, 1, 1>, dim3(n_w + n_c), dim3(kThreads), lds, C.a, W.a, (int)W.grid.x,
               (int)W.grid.y, (int)W.grid.z, (int)C.grid.x);
    else
        cx.run(dgrad_wgrad_f32_k<3, 2, 4, 16, 2, 2>, dim3(n_w + n_c), dim3(kThreads), lds, C.a, W.a, (int)W.grid.x,
               (int)W.grid.y, (int)W.grid.z, (int)C.grid.x);
    return true;
}

}  // namespace rvn
