// Implicit-GEMM convolution (forward and data gradient) on the CDNA4 matrix
// cores, for the units c_k(x) = Conv_kxk(ReLU(BN(x))) of Section 2.2.
//
// GEMM view.  D[ko][pixel] = sum_k Wt[ko][k] * A[k][pixel], k = (c, r, s).
// One v_mfma_f32_16x16x4_f32 multiplies a 16(ko) x 4(k) filter slice by a
// 4(k) x 16(pixel) activation slice; the 4 k-values are 4 consecutive input
// channels at one filter tap.  Output channels sit on the M side so that a
// lane's result register holds consecutive pixels of one channel: results go
// straight to NCHW memory in 64-byte runs, and the skip connection of the
// reversible block (y = r + acc, or x = r - acc when reconstructing,
// Section 3.1) is applied in the same registers.
//
// Work decomposition.  A workgroup (4 wavefronts) owns a band of TH full
// image rows of IMGS images and MT*16 output channels.  Pixels are cut into
// tiles of 16 (1x16 or 2x8); wavefront w takes tiles w, w+4, ...  (NT each).
// The input band (+1 halo row above and below for 3x3) is staged through LDS
// KC channels at a time, NCHW order, rows padded so that the four channel
// planes an instruction reads fall into disjoint banks.  The BN scale/shift
// and ReLU of the unit are applied on the way into LDS, so a(x) never exists
// in HBM; image borders are zero in a(x), not in x, hence the zero fill
// happens after that step.  Filters are staged per chunk in the order the A
// operand consumes them.
//
// With bf16 operands the activation and the filter are rounded to bf16
// (nearest even) on the way into LDS and multiplied by the fp32 matrix
// instruction: identical to a bf16 instruction with fp32 accumulation up to
// summation order.
#include "conv_mfma_body.h"
#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = kConvThreads;

template <int KS, int MT, int NT, int KC, bool EMIT = false>
__global__ __launch_bounds__(kThreads) void conv_mfma_f32_k(const ConvArgs p) {
    extern __shared__ __align__(16) float smem[];
    conv_mfma_f32_body<KS, MT, NT, KC, EMIT>(p, blockIdx.x, blockIdx.y, smem);
}

uint32_t fdiv_magic(int d) { return d == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)d + 1ull); }

int ilog2(int v) {
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

// Choose the band height, images per workgroup and tiles per wavefront.
struct Tiling {
    int TH, IMGS, NT, trows, tcols, ctl, tiles_per_img, n_tiles, bands;
    int lrows, pitch, plane;
    size_t lds_bytes;
};

// LDS geometry for a band of th rows.  Row pitch: a left pad of 4 floats (3x3)
// keeps the 16-byte staging stores aligned and leaves room for the left halo
// column; then the widest pixel tile and the right halo column.  Plane stride
// = 16 mod 32 floats, so that the four channel planes one matrix instruction
// reads (16 consecutive floats each) fall into disjoint LDS banks.
void set_geometry(Tiling &t, int ks, int kc, int mt) {
    const int lp = ks == 3 ? 4 : 0;
    t.lrows = t.TH + ks - 1;
    t.pitch = ((lp + t.ctl * t.tcols + (ks == 3 ? 1 : 0)) + 3) / 4 * 4;
    int plane = t.lrows * t.pitch;
    plane += (16 - plane % 32 + 32) % 32;
    t.plane = plane;
    t.lds_bytes = ((size_t)t.IMGS * kc * plane + (size_t)(kc / 4) * ks * ks * mt * 64) * 4;
}

Tiling choose_tiling(const Geo &g, int ks, int kc, int mt) {
    Tiling best{};
    double best_score = -1.0;
    const int w16 = (g.w + 15) / 16 * 16, w8 = (g.w + 7) / 8 * 8;
    const int tcols = w16 <= w8 ? 16 : 8, trows = 16 / tcols;
    const int ctl = (g.w + tcols - 1) / tcols;
    for (int nt : {4, 7}) {
        const int slots = kWaves * nt;
        for (int imgs : {1, 2, 4, 7, 8}) {
            if (imgs > g.n && imgs != 1) continue;
            for (int th = trows; th <= ((g.h + trows - 1) / trows) * trows; th += trows) {
                if (imgs > 1 && th < g.h) continue;  // several images only when a band is a whole image
                Tiling t{};
                t.TH = th; t.IMGS = imgs; t.NT = nt; t.trows = trows; t.tcols = tcols; t.ctl = ctl;
                t.tiles_per_img = (th / trows) * ctl;
                t.n_tiles = imgs * t.tiles_per_img;
                if (t.n_tiles > slots) break;
                t.bands = (g.h + th - 1) / th;
                set_geometry(t, ks, kc, mt);
                if (t.lds_bytes > 64 * 1024) continue;
                const int groups = (g.n + imgs - 1) / imgs;
                // useful pixels over issued matrix-instruction columns, whole problem
                const double useful = (double)g.n * g.h * g.w;
                const double issued = (double)groups * t.bands * slots * 16;
                double score = useful / issued;
                // prefer enough workgroups to fill 256 CUs twice over
                const double wgs = (double)groups * t.bands;
                if (wgs < 512) score *= 0.5 + 0.5 * wgs / 512;
                if (score > best_score + 1e-9) {
                    best_score = score;
                    best = t;
                }
            }
        }
    }
    return best;
}

template <int KS, int KC>
void launch_conv(Ctx &cx, ConvArgs &a, const Tiling &tl, int mt, dim3 grid) {
#define RVN_CASE(MT_, NT_)                                                                    \
    if (mt == MT_ && tl.NT == NT_) {                                                          \
        cx.run(conv_mfma_f32_k<KS, MT_, NT_, KC>, grid, dim3(kThreads), tl.lds_bytes, a);     \
        return;                                                                               \
    }
    RVN_CASE(1, 4) RVN_CASE(2, 4) RVN_CASE(4, 4)
    RVN_CASE(1, 7) RVN_CASE(2, 7) RVN_CASE(4, 7)
#undef RVN_CASE
}

void conv_mfma(Ctx &cx, View in, const float *scale_shift, const float *w, bool transposed, int ci,
               int co, int ks, Geo g, bool bf16, Epilogue ep, const View *r, View out) {
    ConvLaunch L;
    if (!conv_mfma_plan(in, scale_shift, w, transposed, ci, co, ks, g, bf16, ep, r, out, L)) {
        cx.fail(hipErrorInvalidConfiguration);  // no tiling fits (image rows too wide for LDS)
        return;
    }
    Tiling tl{};
    tl.NT = L.nt;
    tl.lds_bytes = L.lds_bytes;
    ConvArgs a = L.a;
    // Statistics of the output for the BN layer that reads it next (fp32 operands, 3x3, up to 32 output
    // channels, 4 tiles per wavefront): every tile slot of every workgroup must be a whole, valid tile.
    const int tiles = (int)L.grid.x * kWaves;
    const bool whole = a.whole != 0;
    if (cx.want_emit && cx.emit_buf && !bf16 && !transposed && ks == 3 && L.kc == 16 && L.nt == 4 && L.mt <= 2 &&
        whole && (size_t)co * tiles * 2 <= cx.emit_floats) {
        a.emit = cx.emit_buf;
        a.emit_tiles = tiles;
        cx.emitted = EmittedStats{out.p, out.sn, out.sc, co, g.n, g.h, g.w, tiles, 16 * L.nt};
        if (L.mt == 1) cx.run(conv_mfma_f32_k<3, 1, 4, 16, true>, L.grid, dim3(kThreads), tl.lds_bytes, a);
        else cx.run(conv_mfma_f32_k<3, 2, 4, 16, true>, L.grid, dim3(kThreads), tl.lds_bytes, a);
        return;
    }
    if (ks == 3) {
        if (L.kc == 8) launch_conv<3, 8>(cx, a, tl, L.mt, L.grid);
        else launch_conv<3, 16>(cx, a, tl, L.mt, L.grid);
    } else {
        launch_conv<1, 16>(cx, a, tl, L.mt, L.grid);
    }
}

}  // namespace

bool conv_mfma_plan(View in, const float *scale_shift, const float *w, bool transposed, int ci, int co, int ks,
                    Geo g, bool bf16, Epilogue ep, const View *r, View out, ConvLaunch &L) {
    const int mt = co <= 16 ? 1 : co <= 32 ? 2 : 4;
    const int kc = ks == 3 ? (mt == 4 ? 8 : 16) : 16;
    const Tiling tl = choose_tiling(g, ks, kc, mt);
    if (tl.NT == 0) return false;
    if ((int64_t)ci * co * ks * ks >= ((int64_t)1 << 30)) return false;  // filter elements are indexed in 32 bits
    ConvArgs a{};
    a.in = in.p; a.isn = in.sn; a.isc = in.sc;
    a.scale_shift = scale_shift;
    a.w = w;
    a.r = r ? r->p : nullptr; a.rsn = r ? r->sn : 0; a.rsc = r ? r->sc : 0;
    a.out = out.p; a.osn = out.sn; a.osc = out.sc;
    a.N = g.n; a.H = g.h; a.W = g.w; a.CI = ci; a.CO = co;
    a.ep = (int)ep; a.transposed = transposed ? 1 : 0; a.round_bf16 = bf16 ? 1 : 0;
    a.TH = tl.TH; a.IMGS = tl.IMGS; a.bands = tl.bands;
    a.trows = tl.trows; a.tcols_log2 = ilog2(tl.tcols); a.ctl = tl.ctl;
    a.tiles_per_img = tl.tiles_per_img; a.n_tiles = tl.n_tiles;
    a.lrows = tl.lrows; a.pitch = tl.pitch; a.plane = tl.plane;
    a.img_stride = kc * tl.plane;
    a.m_tpi = fdiv_magic(a.tiles_per_img);
    a.m_ctl = fdiv_magic(a.ctl);
    const int64_t lim = (int64_t)1 << 30;
    auto fits = [&](const View &v, int c) {
        return (v.sn & 3) == 0 && (v.sc & 3) == 0 && (reinterpret_cast<uintptr_t>(v.p) & 15) == 0 &&
               (int64_t)g.n * v.sn + (int64_t)c * v.sc + (int64_t)g.h * g.w < lim;
    };
    a.vec32 = (g.w & 3) == 0 && fits(in, ci) && fits(out, co) && (!r || fits(*r, co));
    a.whole = a.n_tiles == kWaves * tl.NT && g.h % a.TH == 0 && a.TH % a.trows == 0 && g.w % (1 << a.tcols_log2) == 0 &&
              g.n % a.IMGS == 0;
    a.tpr_log2 = ilog2((g.w + 3) / 4);
    a.inv_lrows = 1.0f / (float)a.lrows;
    L.a = a;
    L.ks = ks; L.kc = kc; L.mt = mt; L.nt = tl.NT;
    L.grid = dim3((unsigned)(tl.bands * ((g.n + tl.IMGS - 1) / tl.IMGS)), (unsigned)((co + mt * 16 - 1) / (mt * 16)));
    L.lds_bytes = tl.lds_bytes;
    return true;
}

void conv_fwd(Ctx &cx, View x, const float *scale_shift, rvn_dtype dt, const float *w, const uint16_t *wq, int cin,
              int cout, int ks, Geo g, Epilogue ep, const View *r, View out, float *scratch) {
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_fwd_calls += 1;
    cx.cost.conv_flops += flops;
    // (counting mode walks through the dispatch as well: which kernel takes the layer decides whether the
    // next statistics call is a merge of epilogue partials or a pass over the tensor)
    if (!cx.launch(K_CONV_FWD, P * cin * 4.0 + P * cout * 4.0 * (ep == EP_STORE ? 1.0 : 2.0), flops) && !cx.dry) return;
    cx.emitted = EmittedStats{};
    cx.want_emit = true;  // forward convolutions feed a BN layer next: let the kernel describe its output if it can
    if (!(dt == RVN_BF16 && conv_bf16(cx, x, scale_shift, w, wq, false, cin, cout, ks, g, ep, r, out, scratch)))
        conv_mfma(cx, x, scale_shift, w, false, cin, cout, ks, g, dt == RVN_BF16, ep, r, out);
    cx.want_emit = false;
}

void conv_dgrad(Ctx &cx, View dh, rvn_dtype dt, const float *w, const uint16_t *wq, int cin, int cout, int ks,
                Geo g, float *da, float *scratch) {
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_dgrad_calls += 1;
    cx.cost.conv_flops += flops;
    // (counting mode walks through the dispatch: a channel-split launch is followed by a reduce launch)
    if (!cx.launch(K_CONV_DGRAD, P * cout * 4.0 + P * cin * 4.0, flops) && !cx.dry) return;
    // A stride-1 "same" convolution of dh (cout channels) with the transposed,
    // flipped filter, producing cin channels.
    if (dt == RVN_BF16 && conv_bf16(cx, dh, nullptr, w, wq, true, cout, cin, ks, g, EP_STORE, nullptr, dense_view(da, cin, g), scratch))
        return;
    conv_mfma(cx, dh, nullptr, w, true, cout, cin, ks, g, dt == RVN_BF16, EP_STORE, nullptr,
              dense_view(da, cin, g));
}

}  // namespace rvn
