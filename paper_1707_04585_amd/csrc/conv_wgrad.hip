// Filter gradient of the units c_k(x) = Conv_kxk(ReLU(BN(x))) (Section 2.2) on
// the CDNA4 matrix cores: the "ordinary backprop" step of Algorithm 1
// (Section 3.2) that produces the derivative with respect to the weights.
//
// GEMM view.  For every filter tap (r, s):
//     dW[ko][c] = sum_pixels dh[ko][pixel] * a[c][pixel + (r - pad, s - pad)]
// i.e. M = output channels, N = input channels, reduction over all N*H*W
// pixels.  One v_mfma_f32_16x16x4_f32 consumes 4 consecutive pixels of one
// image row: its A operand is a 16(ko) x 4(pixel) slice of dh, its B operand a
// 4(pixel) x 16(c) slice of a, shifted by the tap.
//
// Work decomposition.  The pixels are cut into units (TH full rows of IMGS
// images); workgroup s walks over a contiguous range of units and keeps its
// partial sums in registers, so each workgroup writes its share of dW once.
// Inside a workgroup every wavefront owns one 16x16 (ko, c) tile for all k*k
// taps and a 1/KW share of the 4-pixel steps of a unit.  Both operands are
// staged through LDS in NCHW order: dh as is (rounded to bf16 when the
// convolution works on bf16 operands) and a(x) = max(x*scale + shift, 0)
// formed on the way in from the layer input x, with zero halo rows/columns --
// a(x) is never read from HBM.  The global loads of the next unit are issued
// before the matrix instructions of the current one and land in LDS after
// them.  The workgroups' partial results are summed by a second kernel in a
// fixed order (no floating-point atomics: results are bitwise reproducible).
#include "conv_wgrad_body.h"
#include "kernels.h"
#include "wgrad_reduce.h"

namespace rvn {

namespace {

constexpr int kThreads = kWgradThreads;

template <int KS, int MT, int CT, bool VEC>
__global__ __launch_bounds__(kThreads) void conv_wgrad_mfma_k(const WgradArgs p) {
    extern __shared__ __align__(16) float smem[];
    conv_wgrad_mfma_body<KS, MT, CT, VEC>(p, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.z, smem);
}

__global__ __launch_bounds__(kThreads) void wgrad_reduce_k(const WgradReduce r) {
    __shared__ float lds[kThreads];
    wgrad_reduce_body(r, blockIdx.x, lds);
}

struct WgradPlan {
    int MT, CT, TH, IMGS, bands, units, S, upw, Wq, lrows;
    int a_pitch, a_img, a_plane, d_pitch, d_img, d_plane, a_items, d_items;
    size_t lds_bytes;
    int tiles_ko, tiles_c, part_stride;
    bool ok;
};

uint32_t fdiv_magic(int d) { return d == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)d + 1ull); }


int bank_pad(int plane) {  // smallest value >= plane that is 4 modulo 64
    return plane + ((4 - plane % 64) + 64) % 64;
}

WgradPlan plan_wgrad(int cin, int cout, int ks, const Geo &g) {
    WgradPlan w{};
    w.MT = cout <= 16 ? 1 : 2;
    w.CT = cin <= 16 ? 1 : 2;
    const int lp = ks == 3 ? 4 : 0;
    w.Wq = (g.w + 3) / 4;
    w.a_pitch = lp + 4 * w.Wq + (ks == 3 ? 4 : 0);
    w.d_pitch = 4 * w.Wq;
    w.tiles_ko = (cout + w.MT * 16 - 1) / (w.MT * 16);
    w.tiles_c = (cin + w.CT * 16 - 1) / (w.CT * 16);
    const size_t red_bytes = (size_t)4 * ks * ks * 256 * 4;
    // Largest unit that fits: whole images if possible, else the tallest band.
    auto fits = [&](int th, int imgs) {
        const int lrows = th + ks - 1;
        const int a_img = lrows * w.a_pitch, d_img = th * w.d_pitch;
        const int a_plane = bank_pad(imgs * a_img), d_plane = bank_pad(imgs * d_img);
        const int a_items = w.CT * 16 * imgs * lrows * (w.a_pitch / 4);
        const int d_items = w.MT * 16 * imgs * th * w.Wq;
        const size_t bytes = ((size_t)w.CT * 16 * a_plane + (size_t)w.MT * 16 * d_plane) * 4;
        if (a_items > kItemsA * kThreads || d_items > kItemsD * kThreads || bytes > 64 * 1024 || imgs > 255 || lrows > 4000) return false;
        w.TH = th; w.IMGS = imgs; w.lrows = lrows;
        w.a_img = a_img; w.d_img = d_img; w.a_plane = a_plane; w.d_plane = d_plane;
        w.a_items = a_items; w.d_items = d_items;
        w.lds_bytes = bytes > red_bytes ? bytes : red_bytes;
        return true;
    };
    w.ok = false;
    for (int imgs = g.n < 8 ? g.n : 8; imgs >= 1 && !w.ok; --imgs) w.ok = fits(g.h, imgs);
    for (int th = g.h - 1; th >= 1 && !w.ok; --th) w.ok = fits(th, 1);
    if (!w.ok) return w;
    if (w.IMGS == 1) {  // equal bands: no taller than what fits, as few as that allows
        const int bands = (g.h + w.TH - 1) / w.TH;
        fits((g.h + bands - 1) / bands, 1);
    }
    w.bands = (g.h + w.TH - 1) / w.TH;
    w.units = ((g.n + w.IMGS - 1) / w.IMGS) * w.bands;
    const int groups = w.tiles_ko * w.tiles_c;
    w.part_stride = groups * w.MT * w.CT * ks * ks * 256;
    int s = 256 / groups;  // one workgroup per compute unit
    if (s < 1) s = 1;
    if (s > w.units) s = w.units;
    w.upw = (w.units + s - 1) / s;
    w.S = (w.units + w.upw - 1) / w.upw;
    return w;
}

}  // namespace

size_t wgrad_scratch_floats(int cin, int cout, int ks, const Geo &g) {
    const WgradPlan w = plan_wgrad(cin, cout, ks, g);
    const size_t a = w.ok ? (size_t)w.S * w.part_stride : 0, b = wgrad_bf16_scratch_floats(cin, cout, ks, g);
    return a > b ? a : b;
}

void conv_wgrad(Ctx &cx, View x, const float *scale_shift, rvn_dtype dt, View dh, int cin, int cout,
                int ks, Geo g, float *scratch, float *dw, bool accumulate, WgradReduce *defer) {
    if (defer) defer->blocks = 0;
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_wgrad_calls += 1;
    cx.cost.conv_flops += flops;
    if (dt == RVN_BF16 &&
        conv_wgrad_bf16(cx, x, scale_shift, dh, cin, cout, ks, g, scratch, dw, accumulate,
                        P * cin * 4.0 + P * cout * 4.0, flops, defer))
        return;
    WgradLaunch L;
    WgradReduce red{};
    const bool ok = conv_wgrad_plan(x, scale_shift, dt == RVN_BF16, dh, cin, cout, ks, g, scratch, dw, accumulate, L, red);
    if (cx.launch(K_CONV_WGRAD, P * cin * 4.0 + P * cout * 4.0, flops)) {
        if (!ok) {  // image rows too wide for LDS
            cx.fail(hipErrorInvalidConfiguration);
            return;
        }
        const WgradArgs &a = L.a;
#define RVN_CASE(KS_, MT_, CT_)                                                                        \
    if (ks == KS_ && L.mt == MT_ && L.ct == CT_) {                                                     \
        if (L.vec) cx.run(conv_wgrad_mfma_k<KS_, MT_, CT_, true>, L.grid, dim3(kThreads), L.lds_bytes, a);   \
        else cx.run(conv_wgrad_mfma_k<KS_, MT_, CT_, false>, L.grid, dim3(kThreads), L.lds_bytes, a);      \
    }
        RVN_CASE(3, 1, 1) RVN_CASE(3, 1, 2) RVN_CASE(3, 2, 1) RVN_CASE(3, 2, 2)
        RVN_CASE(1, 1, 1) RVN_CASE(1, 1, 2) RVN_CASE(1, 2, 1) RVN_CASE(1, 2, 2)
#undef RVN_CASE
    }
    if (!ok) return;
    if (defer) *defer = red;
    else wgrad_reduce(cx, red);
}

bool conv_wgrad_plan(View x, const float *scale_shift, bool bf16, View dh, int cin, int cout, int ks, Geo g,
                     float *scratch, float *dw, bool accumulate, WgradLaunch &L, WgradReduce &red) {
    const WgradPlan w = plan_wgrad(cin, cout, ks, g);
    if (!w.ok) return false;
    WgradArgs a{};
    a.x = x.p; a.xsn = x.sn; a.xsc = x.sc;
    a.scale_shift = scale_shift;
    a.dh = dh.p; a.dsn = dh.sn; a.dsc = dh.sc;
    a.part = scratch;
    a.N = g.n; a.H = g.h; a.W = g.w; a.CI = cin; a.CO = cout;
    a.round_bf16 = bf16 ? 1 : 0;
    a.TH = w.TH; a.IMGS = w.IMGS; a.bands = w.bands; a.units = w.units; a.upw = w.upw;
    a.Wq = w.Wq; a.lrows = w.lrows;
    a.a_pitch = w.a_pitch; a.a_img = w.a_img; a.a_plane = w.a_plane;
    a.d_pitch = w.d_pitch; a.d_img = w.d_img; a.d_plane = w.d_plane;
    a.a_items = w.a_items; a.d_items = w.d_items;
    a.steps_per_img = w.TH * w.Wq;
    a.steps = w.IMGS * w.TH * w.Wq;
    a.m_aq = fdiv_magic(w.a_pitch / 4); a.m_lrows = fdiv_magic(w.lrows); a.m_imgs = fdiv_magic(w.IMGS);
    a.m_wq = fdiv_magic(w.Wq); a.m_th = fdiv_magic(w.TH);
    a.part_stride = w.part_stride;
    L.a = a;
    L.ks = ks; L.mt = w.MT; L.ct = w.CT;
    L.grid = dim3((unsigned)w.S, (unsigned)w.tiles_ko, (unsigned)w.tiles_c);
    L.lds_bytes = w.lds_bytes;
    L.vec = (g.w & 3) == 0 && (x.sn & 3) == 0 && (x.sc & 3) == 0 && (dh.sn & 3) == 0 && (dh.sc & 3) == 0 &&
            (reinterpret_cast<uintptr_t>(x.p) & 15) == 0 && (reinterpret_cast<uintptr_t>(dh.p) & 15) == 0;
    red = WgradReduce{};
    red.part = scratch; red.dw = dw;
    red.part_stride = w.part_stride; red.S = w.S; red.KS2 = ks * ks; red.MT = w.MT; red.CT = w.CT;
    red.tiles_c = w.tiles_c; red.CO = cout; red.CI = cin; red.accumulate = accumulate ? 1 : 0;
    red.tile = 16; red.wide = w.S <= 16 ? 1 : 0;
    red.blocks = red.wide ? (w.part_stride + 255) / 256 : (w.part_stride + 31) / 32;
    return true;
}

void wgrad_reduce(Ctx &cx, const WgradReduce &r) {
    if (r.blocks <= 0) return;
    if (cx.launch(K_WGRAD_REDUCE, 0.0)) cx.run(wgrad_reduce_k, dim3((unsigned)r.blocks), dim3(kThreads), 0, r);
}

}  // namespace rvn
