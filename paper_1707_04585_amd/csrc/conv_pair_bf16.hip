// Data gradient and filter gradient of one layer with bf16 operands in a single launch.
//
// Both need only the upstream gradient dh (Algorithm 1: the "ordinary backprop"
// steps), so they are independent.  At the small and late-stage layers neither
// fills the chip on its own (a few dozen to a few hundred workgroups for 512
// workgroup slots), and each pays its own launch and its own ramp; one launch
// holds the workgroups of both, filter gradient first (it has the longer
// dependent chain), so that the two run side by side on the same compute units
// and the load phases of one overlap the matrix phases of the other.  The
// bodies are the ones of the separate kernels, unchanged: results are bit for
// bit those of two launches.
#include <algorithm>

#include "conv1x1_bf16_body.h"
#include "conv3x3_bf16_body.h"
#include "conv_wgrad_bf16_body.h"
#include "conv_wgrad_body.h"
#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;

// Workgroup b < n_w belongs to the filter gradient's grid (w_gx, w_gy, w_gz), x fastest; ids from
// w_real up to n_w (n_w: w_real rounded up to a multiple of 8, so that the convolution's ids keep
// their die) do nothing; the rest is the convolution's grid (c_gx, c_gy, c_gz).
struct PairGrid {
    int w_gx, w_gy, w_gz, w_real, n_w;
    int c_gx, c_gy, c_gz;
};

template <int KS, int MT, int CT, bool VEC>
__device__ __forceinline__ void wgrad_part(const WgArgs &w, const PairGrid &q, int b, uint16_t *smem16) {
    if (b >= q.w_real) return;
    const int bx = b % q.w_gx, t = b / q.w_gx;
    wg::conv_wgrad_bf16_body<KS, MT, CT, VEC>(w, bx, t % q.w_gy, t / q.w_gy, q.w_gz, smem16);
}

template <int MTW, int KC, int NI, int MT, int CT, bool VEC>
__global__ __launch_bounds__(kThreads, 2) void dgrad_wgrad3_bf16_k(const C3Args c, const WgArgs w, const PairGrid q) {
    extern __shared__ __align__(16) uint16_t smem16[];
    const int b = blockIdx.x;
    if (b < q.n_w) {
        wgrad_part<3, MT, CT, VEC>(w, q, b, smem16);
    } else {
        const int i = b - q.n_w;
        const int bx = i % q.c_gx, t = i / q.c_gx;
        c3::conv3x3_bf16_body<1, MTW, 2, KC, false, NI>(c, bx, t % q.c_gy, t / q.c_gy, q.c_gz, smem16);
    }
}

template <int MTW, int DEPTH, bool GEN, int MT, int CT, bool VEC>
__global__ __launch_bounds__(kThreads, 2) void dgrad_wgrad1_bf16_k(const C1Args c, const WgArgs w, const PairGrid q) {
    extern __shared__ __align__(16) uint16_t smem16[];
    const int b = blockIdx.x;
    if (b < q.n_w) wgrad_part<1, MT, CT, VEC>(w, q, b, smem16);
    else c1::conv1x1_bf16_body<MTW, DEPTH, GEN, false>(c, b - q.n_w, q.c_gx, reinterpret_cast<float *>(smem16));
}

// Layers of at most 16 x 16 channels: their filter gradient is the kernel on the fp32 matrix instruction
// (operands rounded to bf16 on the way in), one 16 x 16 tile per workgroup.
template <int NI>
__global__ __launch_bounds__(kThreads, 2) void dgrad3_bf16_wgrad16_k(const C3Args c, const WgradArgs w, const PairGrid q) {
    extern __shared__ __align__(16) uint16_t smem16[];
    const int b = blockIdx.x;
    if (b < q.n_w) {
        if (b >= q.w_real) return;
        const int bx = b % q.w_gx, t = b / q.w_gx;
        conv_wgrad_mfma_body<3, 1, 1, true>(w, bx, t % q.w_gy, t / q.w_gy, q.w_gz, reinterpret_cast<float *>(smem16));
    } else {
        const int i = b - q.n_w;
        const int bx = i % q.c_gx, t = i / q.c_gx;
        c3::conv3x3_bf16_body<1, 1, 2, 16, false, NI>(c, bx, t % q.c_gy, t / q.c_gy, q.c_gz, smem16);
    }
}

// More than 64 KB of dynamic LDS has to be asked for, once per kernel.
template <typename K, typename A, typename B>
bool launch_pair(Ctx &cx, K kernel, bool &raised, unsigned blocks, size_t lds, const A &c, const B &w,
                 const PairGrid &q) {
    if (!raised && !cx.dry && lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        if (e != hipSuccess) {
            cx.fail(e);
            return false;
        }
        raised = true;
    }
    cx.run(kernel, dim3(blocks), dim3(kThreads), lds, c, w, q);
    return true;
}

template <int MTW, int KC, int NI, bool VEC>
void launch3(Ctx &cx, const C3Launch &C, const WgLaunch &W, const PairGrid &q, unsigned blocks, size_t lds) {
#define RVN_CASE(MT_, CT_)                                                                                          \
    if (W.MT == MT_ && W.CT == CT_) {                                                                               \
        static bool raised = false;                                                                                 \
        launch_pair(cx, dgrad_wgrad3_bf16_k<MTW, KC, NI, MT_, CT_, VEC>, raised, blocks, lds, C.a, W.a, q);        \
    }
    RVN_CASE(1, 1) RVN_CASE(1, 2) RVN_CASE(2, 1) RVN_CASE(2, 2)
#undef RVN_CASE
}

template <int MTW, int DEPTH, bool GEN, bool VEC>
void launch1(Ctx &cx, const C1Launch &C, const WgLaunch &W, const PairGrid &q, unsigned blocks, size_t lds) {
#define RVN_CASE(MT_, CT_)                                                                                          \
    if (W.MT == MT_ && W.CT == CT_) {                                                                               \
        static bool raised = false;                                                                                 \
        launch_pair(cx, dgrad_wgrad1_bf16_k<MTW, DEPTH, GEN, MT_, CT_, VEC>, raised, blocks, lds, C.a, W.a, q);    \
    }
    RVN_CASE(1, 1) RVN_CASE(1, 2) RVN_CASE(2, 1) RVN_CASE(2, 2)
#undef RVN_CASE
}

void set_grids(PairGrid &q, dim3 w, dim3 c) {
    q.w_gx = (int)w.x; q.w_gy = (int)w.y; q.w_gz = (int)w.z;
    q.w_real = q.w_gx * q.w_gy * q.w_gz;
    q.n_w = (q.w_real + 7) / 8 * 8;
    q.c_gx = (int)c.x; q.c_gy = (int)c.y; q.c_gz = (int)c.z;
}

// The 3x3 layers the bf16 filter-gradient kernel leaves to the fp32-instruction one.
bool pair_small(Ctx &cx, View x, const float *scale_shift, View dh, const uint16_t *wq_b, int cin, int cout, Geo g,
                float *wgrad_scratch, float *dw, bool accumulate, float *da, float *conv_scratch, WgradReduce *defer) {
    WgradLaunch W;
    WgradReduce red{};
    if (!conv_wgrad_plan(x, scale_shift, true, dh, cin, cout, 3, g, wgrad_scratch, dw, accumulate, W, red)) return false;
    if (W.mt != 1 || W.ct != 1 || !W.vec) return false;
    C3Launch C;
    if (!conv3x3_bf16_plan(dh, nullptr, wq_b, cout, cin, g, EP_STORE, nullptr, dense_view(da, cin, g), conv_scratch, C))
        return false;
    if (C.MTW != 1 || C.KC != 16) return false;
    PairGrid q{};
    set_grids(q, W.grid, C.grid);
    const int64_t blocks = (int64_t)q.n_w + (int64_t)q.c_gx * q.c_gy * q.c_gz;
    if (blocks >= ((int64_t)1 << 31)) return false;
    const size_t lds = std::max(W.lds_bytes, C.lds_bytes);
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * 9;
    cx.cost.conv_dgrad_calls += 1;
    cx.cost.conv_wgrad_calls += 1;
    cx.cost.conv_flops += 2.0 * flops;
    *defer = red;
    if (cx.launch(K_CONV_DGRAD_WGRAD, 2.0 * (P * cin * 4.0 + P * cout * 4.0), 2.0 * flops)) {
        static bool raised[2] = {false, false};
        if (C.NI == 1) launch_pair(cx, dgrad3_bf16_wgrad16_k<1>, raised[0], (unsigned)blocks, lds, C.a, W.a, q);
        else launch_pair(cx, dgrad3_bf16_wgrad16_k<c3::kInItems>, raised[1], (unsigned)blocks, lds, C.a, W.a, q);
    }
    conv3x3_bf16_finish(cx, C, g);
    return true;
}

}  // namespace

bool conv_dgrad_wgrad_bf16(Ctx &cx, View x, const float *scale_shift, View dh, const uint16_t *wq_b, int cin, int cout,
                           int ks, Geo g, float *wgrad_scratch, float *dw, bool accumulate, float *da,
                           float *conv_scratch, WgradReduce *defer) {
    if (!defer || !wq_b || (ks != 1 && ks != 3) || separate_launches()) return false;
    WgLaunch W;
    if (!conv_wgrad_bf16_plan(x, scale_shift, dh, cin, cout, ks, g, wgrad_scratch, dw, accumulate, W))
        return ks == 3 && pair_small(cx, x, scale_shift, dh, wq_b, cin, cout, g, wgrad_scratch, dw, accumulate, da,
                                     conv_scratch, defer);
    // data gradient: a stride-1 "same" convolution of dh (cout channels) with the
    // transposed, flipped filter (prepared in that order in wq_b), producing cin channels
    const View out = dense_view(da, cin, g);
    C3Launch C3;
    C1Launch C1;
    PairGrid q{};
    size_t lds = W.lds_bytes;
    if (ks == 3) {
        if (!conv3x3_bf16_plan(dh, nullptr, wq_b, cout, cin, g, EP_STORE, nullptr, out, conv_scratch, C3)) return false;
        // rows that are not whole 4-pixel groups: instantiated for the wide layers only (64 channels per workgroup, chunks of 16)
        if (!W.vec && (C3.MTW != 2 || C3.KC != 16)) return false;
        set_grids(q, W.grid, C3.grid);
        lds = std::max(lds, C3.lds_bytes);
    } else {
        if (!conv1x1_bf16_plan(dh, nullptr, wq_b, cout, cin, g, EP_STORE, nullptr, out, C1)) return false;
        if (C1.gen && W.vec) return false;  // (planes of H*W % 4 != 0 pixels never have rows of whole 4-pixel groups)
        set_grids(q, W.grid, dim3(C1.wgs));
        lds = std::max(lds, C1.lds_bytes);
    }
    const int64_t blocks = (int64_t)q.n_w + (int64_t)q.c_gx * q.c_gy * q.c_gz;
    if (blocks >= ((int64_t)1 << 31)) return false;

    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_dgrad_calls += 1;
    cx.cost.conv_wgrad_calls += 1;
    cx.cost.conv_flops += 2.0 * flops;
    *defer = W.red;
    if (cx.launch(K_CONV_DGRAD_WGRAD, 2.0 * (P * cin * 4.0 + P * cout * 4.0), 2.0 * flops)) {
        const unsigned nb = (unsigned)blocks;
        if (ks == 3 && W.vec) {
            const int v = (C3.MTW == 2 ? 4 : 0) + (C3.KC == 32 ? 2 : 0) + (C3.NI == 1 ? 1 : 0);
            switch (v) {
                case 0: launch3<1, 16, c3::kInItems, true>(cx, C3, W, q, nb, lds); break;
                case 1: launch3<1, 16, 1, true>(cx, C3, W, q, nb, lds); break;
                case 2: launch3<1, 32, c3::kInItems, true>(cx, C3, W, q, nb, lds); break;
                case 3: launch3<1, 32, 1, true>(cx, C3, W, q, nb, lds); break;
                case 4: launch3<2, 16, c3::kInItems, true>(cx, C3, W, q, nb, lds); break;
                case 5: launch3<2, 16, 1, true>(cx, C3, W, q, nb, lds); break;
                case 6: launch3<2, 32, c3::kInItems, true>(cx, C3, W, q, nb, lds); break;
                default: launch3<2, 32, 1, true>(cx, C3, W, q, nb, lds); break;
            }
        } else if (ks == 3) {
            if (C3.NI == 1) launch3<2, 16, 1, false>(cx, C3, W, q, nb, lds);
            else launch3<2, 16, c3::kInItems, false>(cx, C3, W, q, nb, lds);
        } else if (C1.mtw == 2) {
            if (W.vec) launch1<2, 1, false, true>(cx, C1, W, q, nb, lds);
            else if (C1.gen) launch1<2, 1, true, false>(cx, C1, W, q, nb, lds);
            else launch1<2, 1, false, false>(cx, C1, W, q, nb, lds);
        } else {
            if (W.vec) launch1<1, 2, false, true>(cx, C1, W, q, nb, lds);
            else if (C1.gen) launch1<1, 2, true, false>(cx, C1, W, q, nb, lds);
            else launch1<1, 2, false, false>(cx, C1, W, q, nb, lds);
        }
    }
    if (ks == 3) conv3x3_bf16_finish(cx, C3, g);  // the channel-split data gradient's sum (counted in dry mode too)
    return true;
}

}  // namespace rvn
