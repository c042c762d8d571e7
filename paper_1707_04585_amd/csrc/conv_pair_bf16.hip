// Data gradient and filter gradient of one layer with bf16 operands in a single launch.
//
// Both need only the upstream gradient dh (Algorithm 1: the "ordinary backprop"
// steps), so they are independent.  At the small and late-stage layers neither
// fills the chip on its own (a few dozen to a few hundred workgroups for 512
// workgroup slots), and each pays its own launch and its own ramp; one launch
// holds the workgroups of both, filter gradient first (it has the longer
// dependent chain), so that the two run side by side on the same compute units
// and the load phases of one overlap the matrix phases of the other (which also
// pays at the large layers: the workgroups of a launch otherwise run in step).
// The bodies are the ones of the separate kernels, unchanged: results are bit
// for bit those of two launches.  (Order measured at the 56x56 bottleneck stack:
// filter gradient first 65.4 us per launch, convolution first 72.2, alternating
// groups of eight 88.3.)
//
// DH16 variants: the upstream gradient arrives as bf16 -- the BN backward of the
// layer above wrote it rounded, since both bodies here would round it on load
// anyway -- and is moved to the operand layouts with byte permutes.  Same bits,
// half the bytes of that tensor.
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

template <int KS, int MT, int CT, bool VEC, bool DH16>
__device__ __forceinline__ void wgrad_part(const WgArgs &w, const PairGrid &q, int b, uint16_t *smem16) {
    if (b >= q.w_real) return;
    const int bx = b % q.w_gx, t = b / q.w_gx;
    wg::conv_wgrad_bf16_body<KS, MT, CT, VEC, DH16>(w, bx, t % q.w_gy, t / q.w_gy, q.w_gz, smem16);
}

// DH16: the upstream gradient is bf16 already (written so by the BN backward of the layer above).
template <int MTW, int KC, int NI, int MT, int CT, bool VEC, bool DH16>
__global__ __launch_bounds__(kThreads, 2) void dgrad_wgrad3_bf16_k(const C3Args c, const WgArgs w, const PairGrid q) {
    extern __shared__ __align__(16) uint16_t smem16[];
    const int b = blockIdx.x;
    if (b < q.n_w) {
        wgrad_part<3, MT, CT, VEC, DH16>(w, q, b, smem16);
    } else {
        const int i = b - q.n_w;
        const int bx = i % q.c_gx, t = i / q.c_gx;
        c3::conv3x3_bf16_body<1, MTW, 2, KC, false, NI, DH16>(c, bx, t % q.c_gy, t / q.c_gy, q.c_gz, smem16);
    }
}

template <int MTW, int DEPTH, bool GEN, int MT, int CT, bool VEC, bool DH16>
__global__ __launch_bounds__(kThreads, 2) void dgrad_wgrad1_bf16_k(const C1Args c, const WgArgs w, const PairGrid q) {
    extern __shared__ __align__(16) uint16_t smem16[];
    const int b = blockIdx.x;
    if (b < q.n_w) wgrad_part<1, MT, CT, VEC, DH16>(w, q, b, smem16);
    else c1::conv1x1_bf16_body<MTW, DEPTH, GEN, false, DH16>(c, b - q.n_w, q.c_gx, reinterpret_cast<float *>(smem16));
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

template <int MTW, int KC, int NI, bool VEC, bool DH16>
void launch3(Ctx &cx, const C3Launch &C, const WgLaunch &W, const PairGrid &q, unsigned blocks, size_t lds) {
#define RVN_CASE(MT_, CT_)                                                                                          \
    if (W.MT == MT_ && W.CT == CT_) {                                                                               \
        static bool raised = false;                                                                                 \
        launch_pair(cx, dgrad_wgrad3_bf16_k<MTW, KC, NI, MT_, CT_, VEC, DH16>, raised, blocks, lds, C.a, W.a, q);        \
    }
    RVN_CASE(1, 1) RVN_CASE(1, 2) RVN_CASE(2, 1) RVN_CASE(2, 2)
#undef RVN_CASE
}

template <int MTW, int DEPTH, bool GEN, bool VEC, bool DH16>
void launch1(Ctx &cx, const C1Launch &C, const WgLaunch &W, const PairGrid &q, unsigned blocks, size_t lds) {
#define RVN_CASE(MT_, CT_)                                                                                          \
    if (W.MT == MT_ && W.CT == CT_) {                                                                               \
        static bool raised = false;                                                                                 \
        launch_pair(cx, dgrad_wgrad1_bf16_k<MTW, DEPTH, GEN, MT_, CT_, VEC, DH16>, raised, blocks, lds, C.a, W.a, q);    \
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

namespace {

struct PairPlan {
    WgLaunch W;
    C3Launch C3;
    C1Launch C1;
    PairGrid q;
    size_t lds;
    int64_t blocks;
};

// Both tilings of a layer's gradients; false if one of the kernels does not take the layer (or the
// combination has no instance).
bool plan_pair(View x, const float *scale_shift, View dh, const uint16_t *wq_b, int cin, int cout, int ks, Geo g,
               float *wgrad_scratch, float *dw, bool accumulate, float *da, float *conv_scratch, PairPlan &P) {
    if (!conv_wgrad_bf16_plan(x, scale_shift, dh, cin, cout, ks, g, wgrad_scratch, dw, accumulate, P.W)) return false;
    // data gradient: a stride-1 "same" convolution of dh (cout channels) with the
    // transposed, flipped filter (prepared in that order in wq_b), producing cin channels
    const View out = dense_view(da, cin, g);
    P.q = PairGrid{};
    P.lds = P.W.lds_bytes;
    if (ks == 3) {
        if (!conv3x3_bf16_plan(dh, nullptr, wq_b, cout, cin, g, EP_STORE, nullptr, out, conv_scratch, P.C3)) return false;
        // rows that are not whole 4-pixel groups: instantiated for the wide layers only (64 channels per workgroup, chunks of 16)
        if (!P.W.vec && (P.C3.MTW != 2 || P.C3.KC != 16)) return false;
        set_grids(P.q, P.W.grid, P.C3.grid);
        P.lds = std::max(P.lds, P.C3.lds_bytes);
    } else {
        if (!conv1x1_bf16_plan(dh, nullptr, wq_b, cout, cin, g, EP_STORE, nullptr, out, P.C1)) return false;
        if (P.C1.gen && P.W.vec) return false;  // (planes of H*W % 4 != 0 pixels never have rows of whole 4-pixel groups)
        set_grids(P.q, P.W.grid, dim3(P.C1.wgs));
        P.lds = std::max(P.lds, P.C1.lds_bytes);
    }
    P.blocks = (int64_t)P.q.n_w + (int64_t)P.q.c_gx * P.q.c_gy * P.q.c_gz;
    return P.blocks < ((int64_t)1 << 31);
}

template <bool DH16>
void launch_planned(Ctx &cx, int ks, const PairPlan &P) {
    const WgLaunch &W = P.W;
    const unsigned nb = (unsigned)P.blocks;
    if (ks == 3 && W.vec) {
        const C3Launch &C3 = P.C3;
        const int v = (C3.MTW == 2 ? 4 : 0) + (C3.KC == 32 ? 2 : 0) + (C3.NI == 1 ? 1 : 0);
        switch (v) {
            case 0: launch3<1, 16, c3::kInItems, true, DH16>(cx, C3, W, P.q, nb, P.lds); break;
            case 1: launch3<1, 16, 1, true, DH16>(cx, C3, W, P.q, nb, P.lds); break;
            case 2: launch3<1, 32, c3::kInItems, true, DH16>(cx, C3, W, P.q, nb, P.lds); break;
            case 3: launch3<1, 32, 1, true, DH16>(cx, C3, W, P.q, nb, P.lds); break;
            case 4: launch3<2, 16, c3::kInItems, true, DH16>(cx, C3, W, P.q, nb, P.lds); break;
            case 5: launch3<2, 16, 1, true, DH16>(cx, C3, W, P.q, nb, P.lds); break;
            case 6: launch3<2, 32, c3::kInItems, true, DH16>(cx, C3, W, P.q, nb, P.lds); break;
            default: launch3<2, 32, 1, true, DH16>(cx, C3, W, P.q, nb, P.lds); break;
        }
    } else if (ks == 1 && W.vec) {
        if (P.C1.mtw == 2) launch1<2, 1, false, true, DH16>(cx, P.C1, W, P.q, nb, P.lds);
        else launch1<1, 2, false, true, DH16>(cx, P.C1, W, P.q, nb, P.lds);
    } else if constexpr (!DH16) {
        if (ks == 3) {
            if (P.C3.NI == 1) launch3<2, 16, 1, false, false>(cx, P.C3, W, P.q, nb, P.lds);
            else launch3<2, 16, c3::kInItems, false, false>(cx, P.C3, W, P.q, nb, P.lds);
        } else if (P.C1.mtw == 2) {
            if (P.C1.gen) launch1<2, 1, true, false, false>(cx, P.C1, W, P.q, nb, P.lds);
            else launch1<2, 1, false, false, false>(cx, P.C1, W, P.q, nb, P.lds);
        } else {
            if (P.C1.gen) launch1<1, 2, true, false, false>(cx, P.C1, W, P.q, nb, P.lds);
            else launch1<1, 2, false, false, false>(cx, P.C1, W, P.q, nb, P.lds);
        }
    }
}

}  // namespace

bool conv_dgrad_wgrad_takes_bf16_dh(View x, const uint16_t *dh16, const uint16_t *wq_b, int cin, int cout, int ks, Geo g,
                                    float *wgrad_scratch, float *da, float *conv_scratch) {
    if (!wq_b || !dh16 || (ks != 1 && ks != 3) || separate_launches()) return false;
    PairPlan P;
    const View dh = dense_view(reinterpret_cast<float *>(const_cast<uint16_t *>(dh16)), cout, g);
    // (the filter-gradient output plays no part in the tiling)
    if (!plan_pair(x, nullptr, dh, wq_b, cin, cout, ks, g, wgrad_scratch, nullptr, false, da, conv_scratch, P)) return false;
    return P.W.vec && (ks == 3 || !P.C1.gen);
}

bool conv_dgrad_wgrad_bf16(Ctx &cx, View x, const float *scale_shift, View dh, const uint16_t *dh16, const uint16_t *wq_b,
                           int cin, int cout, int ks, Geo g, float *wgrad_scratch, float *dw, bool accumulate,
                           float *da, float *conv_scratch, WgradReduce *defer) {
    if (!defer || !wq_b || (ks != 1 && ks != 3) || separate_launches()) return false;
    if (dh16) dh = dense_view(reinterpret_cast<float *>(const_cast<uint16_t *>(dh16)), cout, g);
    PairPlan P;
    if (!plan_pair(x, scale_shift, dh, wq_b, cin, cout, ks, g, wgrad_scratch, dw, accumulate, da, conv_scratch, P)) {
        WgLaunch W;  // the 3x3 layers the bf16 filter-gradient kernel leaves to the fp32-instruction one
        return !dh16 && ks == 3 && !conv_wgrad_bf16_plan(x, scale_shift, dh, cin, cout, ks, g, wgrad_scratch, dw, accumulate, W) &&
               pair_small(cx, x, scale_shift, dh, wq_b, cin, cout, g, wgrad_scratch, dw, accumulate, da, conv_scratch, defer);
    }
    if (dh16 && !(P.W.vec && (ks == 3 || !P.C1.gen))) return false;  // (the caller asked conv_dgrad_wgrad_takes_bf16_dh first)

    const double Pix = (double)g.pixels();
    const double flops = 2.0 * Pix * cin * cout * ks * ks;
    cx.cost.conv_dgrad_calls += 1;
    cx.cost.conv_wgrad_calls += 1;
    cx.cost.conv_flops += 2.0 * flops;
    *defer = P.W.red;
    // a(x) read and da written in fp32; dh read by both bodies, in 2 or 4 bytes per element
    if (cx.launch(K_CONV_DGRAD_WGRAD, 2.0 * Pix * cin * 4.0 + 2.0 * Pix * cout * (dh16 ? 2.0 : 4.0), 2.0 * flops)) {
        if (dh16) launch_planned<true>(cx, ks, P);
        else launch_planned<false>(cx, ks, P);
    }
    if (ks == 3) conv3x3_bf16_finish(cx, P.C3, g);  // the channel-split data gradient's sum (counted in dry mode too)
    return true;
}

}  // namespace rvn
