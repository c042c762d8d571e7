// Filter gradient with bf16 operands on the CDNA4 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation): the "ordinary backprop" step of
// Algorithm 1 (Section 3.2) that produces the derivative with respect to the
// weights, when the block descriptor asks for bf16 convolution operands.
//
// GEMM view.  For every filter tap (r, s):
//     dW[ko][c] = sum_pixels dh[ko][pixel] * a[c][pixel + (r - pad, s - pad)]
// M = output channels, N = input channels, reduction over all N*H*W pixels.
// One matrix instruction consumes 16 pixels: each lane feeds 8 consecutive
// pixels of one image row for its channel, so both operands live in LDS as
// bf16 NCHW planes (pixel innermost) cut into chunks of 8 pixels, and a chunk
// is one aligned 16-byte read.  A tap that moves one column left or right would
// need a misaligned chunk; it is assembled in registers instead from the
// aligned chunk and one dword of its neighbour (four funnel shifts), so the
// activation tile is stored once, with 8 zero elements before and after every
// row for the halo columns.
//
// Work decomposition as in the fp32 kernel: units of TH full rows of IMGS
// images; workgroup s walks over a contiguous range of units with its partial
// sums in registers; every wavefront owns one 32x32 (ko, c) tile for all k*k
// taps and a 1/KW share of the 16-pixel steps; a(x) = max(x*scale + shift, 0) is
// formed (and rounded to bf16) on the way into LDS.  Partial results are summed
// in a fixed order by wgrad_reduce_body, in a launch of its own or carried by
// another kernel.
#include <algorithm>

#include "conv_wgrad_bf16_body.h"
#include "kernels.h"

namespace rvn {

namespace {

using namespace wg;

template <int KS, int MT, int CT, bool VEC>
__global__ __launch_bounds__(kThreads, 2) void conv_wgrad_bf16_k(const WgArgs p) {
    extern __shared__ __align__(16) uint16_t smem16[];
    conv_wgrad_bf16_body<KS, MT, CT, VEC>(p, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.z, smem16);
}

struct WgPlan {
    int MT, CT, TH, IMGS, bands, units, S, upw, Wq, cpr, lrows;
    int a_pitch, a_img, a_plane, d_pitch, d_img, d_plane, a_items, d_items;
    size_t lds_bytes;
    int tiles_ko, tiles_c, part_stride;
    bool ok;
    Geo g;  // the geometry the plan is for (see wg_geometry)
};

uint32_t fdiv_magic(int d) { return d == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)d + 1ull); }

// Smallest value >= plane that is 8 modulo 16 (elements): planes an odd multiple
// of 16 bytes apart put the 16-byte reads of 8 neighbouring lanes on distinct banks.
int bank_pad(int plane) { return plane + ((8 - plane % 16) + 16) % 16; }

WgPlan plan_wg_tiles(int cin, int cout, int ks, const Geo &g, int ct_max) {
    WgPlan w{};
    w.ok = false;
    if (g.w < 4) return w;  // staging loads 4 pixels of a row at a time
    // A 16 x 16 filter fills a quarter of a 32 x 32 result tile; the fp32-instruction
    // kernel (16 x 16 tiles, operands rounded to bf16 on the way in) is faster there.
    if (cin <= 16 && cout <= 16) return w;
    w.MT = cout <= 32 ? 1 : 2;
    w.CT = cin <= 32 || ct_max < 2 ? 1 : 2;
    w.Wq = (g.w + 3) / 4;
    w.cpr = (g.w + 7) / 8;
    w.a_pitch = ks == 3 ? 8 + w.cpr * 8 + 8 : w.cpr * 8;  // 3x3: 8 zero elements before and after every row
    w.d_pitch = w.cpr * 8;
    w.tiles_ko = (cout + w.MT * 32 - 1) / (w.MT * 32);
    w.tiles_c = (cin + w.CT * 32 - 1) / (w.CT * 32);
    const size_t red_bytes = (size_t)4 * 1024 * 4;
    // Largest unit that fits: whole images if possible, else the tallest band.
    auto fits = [&](int th, int imgs) {
        const int lrows = th + ks - 1;
        const int a_img = lrows * w.a_pitch, d_img = th * w.d_pitch;
        const int a_plane = bank_pad(imgs * a_img), d_plane = bank_pad(imgs * d_img);
        const int a_items = w.CT * 32 * imgs * lrows * w.Wq;
        const int d_items = w.MT * 32 * imgs * th * w.Wq;
        const size_t bytes = ((size_t)w.CT * 32 * a_plane + (size_t)w.MT * 32 * d_plane) * 2;
        // (64 KB: two workgroups per compute unit would hold 78 KB each, but the taller units that buys -- 3 rows
        // for 5 staged instead of 2 for 4 at 56 columns and 64 + 64 channels -- leave 406 slices for 512 slots
        // and fewer units per slice to pipeline: the shared gradient launch took 77.9 us against 65.7)
        if (bytes > 64 * 1024 || imgs > 255 || lrows > 4000) return false;
        if (imgs * lrows * w.Wq > 128) return false;  // staging: at most two 4-pixel items per lane and channel plane
        w.TH = th; w.IMGS = imgs; w.lrows = lrows;
        w.a_img = a_img; w.d_img = d_img; w.a_plane = a_plane; w.d_plane = d_plane;
        w.a_items = a_items; w.d_items = d_items;
        w.lds_bytes = bytes > red_bytes ? bytes : red_bytes;
        return true;
    };
    w.ok = false;
    for (int imgs = g.n < 16 ? g.n : 16; imgs >= 1 && !w.ok; --imgs) w.ok = fits(g.h, imgs);
    for (int th = g.h - 1; th >= 1 && !w.ok; --th) w.ok = fits(th, 1);
    if (!w.ok) return w;
    if (w.IMGS == 1) {  // equal bands: no taller than what fits, as few as that allows
        const int bands = (g.h + w.TH - 1) / w.TH;
        fits((g.h + bands - 1) / bands, 1);
    }
    w.bands = (g.h + w.TH - 1) / w.TH;
    w.units = ((g.n + w.IMGS - 1) / w.IMGS) * w.bands;
    const int groups = w.tiles_ko * w.tiles_c;
    w.part_stride = groups * w.MT * w.CT * ks * ks * 1024;
    // Two workgroups per compute unit (512 in all: 384 measured the same, 768 and 1024 4-10 % slower per
    // launch; half and a quarter were slower on every workload).
    int s = 512 / groups;
    if (s < 1) s = 1;
    if (s > w.units) s = w.units;
    w.upw = (w.units + s - 1) / s;
    w.S = (w.units + w.upw - 1) / w.upw;
    return w;
}

// 64 x 64 tiles per workgroup; for a 3x3 layer with more units than slices to give them to, 64 x 32: the
// same 512 workgroups then write half the partial results (a workgroup's partial filter is its whole
// tile times nine taps, whatever it summed over) for one more read of the upstream gradient, which the
// tile groups of a slice share in their die's L2.  Measured at the 56x56 bottleneck stack: step 15.98 ->
// 15.82 ms, the four-stage body 14.81 -> 14.50; 32 x 32, 32 x 64 and any split of the 1x1 layers were
// slower, and so was the split on the small layers whose slices are limited by their units.
// A 1x1 filter's gradient has no spatial structure: where the rows are not whole 4-pixel groups but the
// planes are (14x14), an image is taken as one row of h*w pixels, which puts the layer on the aligned
// staging path (16-byte loads, whole-unit prefetch, bf16 upstream gradient).
Geo wg_geometry(int ks, const Geo &g) {
    if (ks == 1 && (g.w & 3) != 0 && ((int64_t)g.h * g.w) % 4 == 0 && (int64_t)g.h * g.w <= 512) return Geo{g.n, 1, g.h * g.w};
    return g;
}

WgPlan plan_wg_for(int cin, int cout, int ks, const Geo &g) {
    WgPlan w = plan_wg_tiles(cin, cout, ks, g, 2);
    w.g = g;
    if (!w.ok || ks != 3 || w.CT != 2 || w.units <= 512 / (w.tiles_ko * w.tiles_c)) return w;
    WgPlan n = plan_wg_tiles(cin, cout, ks, g, 1);
    n.g = g;
    return n.ok ? n : w;
}

WgPlan plan_wg(int cin, int cout, int ks, const Geo &g_layer) {
    const Geo flat = wg_geometry(ks, g_layer);
    if (flat.h != g_layer.h) {
        const WgPlan w = plan_wg_for(cin, cout, ks, flat);
        if (w.ok) return w;  // (else the one-row image does not fit a unit: the layer's own rows)
    }
    return plan_wg_for(cin, cout, ks, g_layer);
}

}  // namespace

size_t wgrad_bf16_scratch_floats(int cin, int cout, int ks, const Geo &g) {
    const WgPlan w = plan_wg(cin, cout, ks, g);
    return w.ok ? (size_t)w.S * w.part_stride : 0;
}

bool conv_wgrad_bf16_plan(View x, const float *scale_shift, View dh, int cin, int cout, int ks, Geo g_layer, float *scratch,
                          float *dw, bool accumulate, WgLaunch &L) {
    const WgPlan w = plan_wg(cin, cout, ks, g_layer);
    const Geo g = w.g;
    if (!w.ok) return false;
    // a lane's item offsets (image, row, column within a channel plane of a unit) are 32-bit
    if ((int64_t)w.IMGS * std::max(x.sn, dh.sn) + (int64_t)(w.lrows + 1) * g.w >= ((int64_t)1 << 30)) return false;
    WgArgs a{};
    a.x = x.p; a.xsn = x.sn; a.xsc = x.sc;
    a.scale_shift = scale_shift;
    a.dh = dh.p; a.dsn = dh.sn; a.dsc = dh.sc;
    a.part = scratch;
    a.N = g.n; a.H = g.h; a.W = g.w; a.CI = cin; a.CO = cout;
    a.TH = w.TH; a.IMGS = w.IMGS; a.bands = w.bands; a.units = w.units; a.upw = w.upw;
    a.Wq = w.Wq; a.cpr = w.cpr; a.lrows = w.lrows;
    a.a_pitch = w.a_pitch; a.a_img = w.a_img; a.a_plane = w.a_plane;
    a.d_pitch = w.d_pitch; a.d_img = w.d_img; a.d_plane = w.d_plane;
    a.chunks = w.IMGS * w.TH * w.cpr;
    a.m_wq = fdiv_magic(w.Wq);
    a.part_stride = w.part_stride;
    L.a = a;
    L.KS = ks; L.MT = w.MT; L.CT = w.CT;
    L.grid = dim3((unsigned)w.S, (unsigned)w.tiles_ko, (unsigned)w.tiles_c);
    L.lds_bytes = w.lds_bytes;
    L.vec = (g.w & 3) == 0 && (x.sn & 3) == 0 && (x.sc & 3) == 0 && (dh.sn & 3) == 0 && (dh.sc & 3) == 0 &&
            (reinterpret_cast<uintptr_t>(x.p) & 15) == 0 && (reinterpret_cast<uintptr_t>(dh.p) & 15) == 0;
    WgradReduce red{};
    red.part = scratch; red.dw = dw;
    red.part_stride = w.part_stride; red.S = w.S; red.KS2 = ks * ks; red.MT = w.MT; red.CT = w.CT;
    red.tiles_c = w.tiles_c; red.CO = cout; red.CI = cin; red.accumulate = accumulate ? 1 : 0;
    red.tile = 32; red.wide = w.S <= 16 ? 1 : 0;
    red.blocks = red.wide ? (w.part_stride + 255) / 256 : (w.part_stride + 31) / 32;
    L.red = red;
    return true;
}

bool conv_wgrad_bf16(Ctx &cx, View x, const float *scale_shift, View dh, int cin, int cout, int ks, Geo g,
                     float *scratch, float *dw, bool accumulate, double bytes, double flops, WgradReduce *defer) {
    WgLaunch L;
    if (!conv_wgrad_bf16_plan(x, scale_shift, dh, cin, cout, ks, g, scratch, dw, accumulate, L)) return false;
    if (cx.launch(K_CONV_WGRAD, bytes, flops)) {
#define RVN_CASE(KS_, MT_, CT_)                                                                           \
    if (ks == KS_ && L.MT == MT_ && L.CT == CT_) {                                                        \
        if (L.vec) cx.run(conv_wgrad_bf16_k<KS_, MT_, CT_, true>, L.grid, dim3(kThreads), L.lds_bytes, L.a); \
        else cx.run(conv_wgrad_bf16_k<KS_, MT_, CT_, false>, L.grid, dim3(kThreads), L.lds_bytes, L.a);     \
    }
        RVN_CASE(3, 1, 1) RVN_CASE(3, 1, 2) RVN_CASE(3, 2, 1) RVN_CASE(3, 2, 2)
        RVN_CASE(1, 1, 1) RVN_CASE(1, 1, 2) RVN_CASE(1, 2, 1) RVN_CASE(1, 2, 2)
#undef RVN_CASE
    }
    if (defer) *defer = L.red;
    else wgrad_reduce(cx, L.red);
    return true;
}

}  // namespace rvn
