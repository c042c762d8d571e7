// 3x3 convolution (forward and data gradient) with bf16 operands on the CDNA4
// matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation), for the 3x3 units
// c_3(x) = Conv_3x3(ReLU(BN(x))) of Section 2.2 when the block descriptor asks
// for bf16 convolution operands.
//
// GEMM view.  D[ko][pixel] = sum_{tap, c} Wt[ko][tap][c] * A[c][pixel + tap],
// one matrix instruction per (tap, 16 input channels).  Both operands live in
// LDS with the channel innermost (pixel records and (ko, tap) records of KC + 8
// bf16), so every operand read is one 16-byte access per lane.
//
// What this kernel adds to that scheme:
//  * register tiling: a wavefront owns MTW x NTW tiles of 32 x 32 results, so
//    an LDS read feeds NTW (filter) or MTW (activation) matrix instructions;
//  * software pipelining: the global loads of the next channel chunk (the next
//    two, where a thread holds one staging item; activations as fp32, filter as
//    prepared bf16) are issued before the matrix instructions of chunk i and
//    are converted and written to LDS after them;
//  * staging by linear quads: an item is 4 consecutive pixels of the band's
//    contiguous range in the image plane, times 8 channels, so the loads are
//    16 bytes whatever the image width; BN scale/shift, ReLU and the bf16
//    rounding happen on the way into LDS;
//  * optional split of the input channels over gridDim.z: partial tiles go to
//    scratch and a second kernel sums them in a fixed order and applies the
//    coupling y = r + conv / reconstruction x = r - conv of Section 3.1
//    (otherwise that is done in the accumulator registers here);
//  * an epilogue through buffer resources (scalar channel offsets, one uniform
//    bound check), and workgroup ids remapped so that a die gets a contiguous
//    range of bands (neighbouring bands share input rows).
#include <algorithm>

#include "conv3x3_bf16_body.h"
#include "kernels.h"

namespace rvn {

namespace {

using namespace c3;

template <int WM, int MTW, int NTW, int KC, bool EMIT = false, int NI = kInItems>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_bf16_k(const C3Args p) {
    extern __shared__ __align__(16) uint16_t smem16[];
    conv3x3_bf16_body<WM, MTW, NTW, KC, EMIT, NI>(p, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.z, smem16);
}

// out = ep(r, sum_s part[s]) over dense partial tiles [S][n][c][hw], summed in
// the order s = 0, 1, ...  EMIT (host: h*w a multiple of 64, total a multiple of
// the workgroup size, so a wavefront holds 64 consecutive pixels of one plane):
// the wavefront also leaves the mean and centred sum of squares of what it
// stores at emit[(c * emit_tiles + n * (h*w / 64) + pixel / 64) * 2], for the
// BN layer that reads the tensor next.
template <bool EMIT>
__global__ __launch_bounds__(kThreads) void splitk_reduce_k(const float *__restrict__ part, int64_t part_stride, int S,
                                                            int C, int HW, int64_t total, const float *r,
                                                            int64_t rsn, int64_t rsc, float *out, int64_t osn,
                                                            int64_t osc, int ep, float *emit, int emit_tiles) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    float v = part[i];
    for (int s = 1; s < S; ++s) v += part[(int64_t)s * part_stride + i];
    const int64_t plane = i / HW;
    const int pix = (int)(i - plane * HW);
    const int64_t n = plane / C;
    const int c = (int)(plane - n * C);
    if (ep != EP_STORE) {
        const float rv = r[n * rsn + (int64_t)c * rsc + pix];
        v = ep == EP_ADD ? rv + v : rv - v;
    }
    out[n * osn + (int64_t)c * osc + pix] = v;
    if constexpr (EMIT) {
        const float pivot = __shfl(v, 0, 64);
        float a = v - pivot, b = a * a;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            a += __shfl_xor(a, off, 64);
            b += __shfl_xor(b, off, 64);
        }
        if ((threadIdx.x & 63) == 0) {
            const float mean = pivot + a * (1.f / 64.f);
            const float m2 = fmaxf(b - a * a * (1.f / 64.f), 0.f);
            const int tile = (int)n * (HW >> 6) + (pix >> 6);
            reinterpret_cast<float2 *>(emit)[(int64_t)c * emit_tiles + tile] = make_float2(mean, m2);
        }
    }
}

struct C3Plan {
    int WM, MTW, NTW, KC, TR, IMGS, bands, lrows, lcols, q_per_img, in_items, chunks, S, cps;
    size_t lds_bytes;
    bool ok;
};

C3Plan plan_c3(int ci, int co, const Geo &g, int stride = 1) {
    C3Plan pl{};
    pl.ok = false;
    if (ci % 8 != 0 || g.w < 4 || ci > 4096) return pl;
    if (stride != 1 && (stride != 2 || g.h % 2 || g.w % 2)) return pl;
    const int oh = g.h / stride, ow = g.w / stride;  // the result's rows and columns
    // Output channels per workgroup and the wavefront arrangement.
    // 64 output channels per workgroup at most, the four wavefronts side by side along the pixels: with
    // 128 channels (two wavefronts stacked) the wide layers were 5-10 % slower (twice the filter tile per
    // workgroup, half as many pixel slots).
    pl.WM = 1; pl.MTW = co <= 32 ? 1 : 2; pl.NTW = 2;
    const int ch = pl.WM * pl.MTW * 32, slots = (4 / pl.WM) * pl.NTW * 32;
    // One chunk of 32 channels when that is the whole input; otherwise chunks of
    // 16, which pipeline better (measured on 64-, 56- and 32-channel layers).
    pl.KC = ci == 32 && ch <= 64 ? 32 : 16;
    const int rec = pl.KC + kPadK, octs = pl.KC / 8;
    // Pixel block: the fullest block of whole rows (or whole images) that fits.
    double best = -1.0;
    for (int imgs = 1; imgs <= 16 && imgs <= g.n; ++imgs) {
        for (int tr = imgs > 1 ? oh : 1; tr <= oh; ++tr) {
            const int npix = imgs * tr * ow;
            if (npix > slots) break;
            const int lrows = stride * (tr - 1) + 3, lcols = g.w + 2;
            const int q = (lrows * g.w + 3) / 4;
            const int items = imgs * q * octs;
            const size_t bytes = ((size_t)imgs * lrows * lcols + (size_t)ch * 9) * rec * 2 + (size_t)ci * 8;
            if (items > kInItems * kThreads || bytes > 76 * 1024) break;
            const int bands = (oh + tr - 1) / tr, groups = (g.n + imgs - 1) / imgs;
            const double useful = (double)g.n * oh * ow, issued = (double)groups * bands * slots;
            const double score = useful / issued;
            if (score > best) {
                best = score;
                pl.TR = tr; pl.IMGS = imgs; pl.bands = bands; pl.lrows = lrows; pl.lcols = lcols;
                pl.q_per_img = q; pl.in_items = items; pl.lds_bytes = bytes;
                pl.ok = true;
            }
        }
    }
    if (!pl.ok) return pl;
    pl.chunks = (ci + pl.KC - 1) / pl.KC;
    const int64_t wgs = (int64_t)((g.n + pl.IMGS - 1) / pl.IMGS) * pl.bands * ((co + ch - 1) / ch);
    pl.S = 1;
    // Too few workgroups for the chip (measured: at most one per two compute
    // units): split the input channels over gridDim.z as well.  (56 -> 56 channels at 8x8, N=128: the
    // 32 unsplit workgroups take 18.5 us, the 64 split ones 10.1 us plus 4.2 us for the sum.)
    if (wgs <= 128 && pl.chunks >= 4) pl.S = (int)std::min<int64_t>(pl.chunks / 2, (512 + wgs - 1) / wgs);
    pl.cps = (pl.chunks + pl.S - 1) / pl.S;
    pl.S = (pl.chunks + pl.cps - 1) / pl.cps;
    return pl;
}

// More than 64 KB of dynamic LDS has to be asked for, once per kernel.
template <typename K>
bool raise_lds_limit(Ctx &cx, K kernel, bool &raised) {
    if (raised || cx.dry) return true;
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
    if (e != hipSuccess) {
        cx.fail(e);
        return false;
    }
    raised = true;
    return true;
}

template <int WM, int MTW, int NTW, int KC, bool EMIT, int NI>
void launch_c3_items(Ctx &cx, const C3Launch &L, dim3 grid) {
    static bool raised = false;
    if (!raise_lds_limit(cx, conv3x3_bf16_k<WM, MTW, NTW, KC, EMIT, NI>, raised)) return;
    cx.run(conv3x3_bf16_k<WM, MTW, NTW, KC, EMIT, NI>, grid, dim3(kThreads), L.lds_bytes, L.a);
}

template <int WM, int MTW, int NTW, int KC, bool EMIT>
void launch_c3_variant(Ctx &cx, const C3Launch &L, dim3 grid) {
    if (L.NI == 1) launch_c3_items<WM, MTW, NTW, KC, EMIT, 1>(cx, L, grid);
    else launch_c3_items<WM, MTW, NTW, KC, EMIT, kInItems>(cx, L, grid);
}

template <int WM, int MTW, int NTW, int KC>
void launch_c3(Ctx &cx, const C3Launch &L, dim3 grid) {
    if (L.a.emit) launch_c3_variant<WM, MTW, NTW, KC, true>(cx, L, grid);
    else launch_c3_variant<WM, MTW, NTW, KC, false>(cx, L, grid);
}

}  // namespace

bool conv3x3_bf16_ok(int ci, int co, const Geo &g) { return plan_c3(ci, co, g).ok; }

size_t conv3x3_bf16_scratch_floats(int ci, int co, const Geo &g, int stride) {
    const C3Plan pl = plan_c3(ci, co, g, stride);
    return pl.ok && pl.S > 1 ? (size_t)pl.S * g.n * co * (g.h / stride) * (g.w / stride) : 0;
}

bool conv3x3_bf16_plan(View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g, Epilogue ep,
                       const View *r, View out, float *scratch, C3Launch &L, int stride) {
    if (!wq) return false;
    const C3Plan pl = plan_c3(ci, co, g, stride);
    const int oh = g.h / stride, ow = g.w / stride;  // `out`, `r` and the partial tiles have the result's geometry
    if (!pl.ok || (pl.S > 1 && !scratch)) return false;
    if (pl.WM != 1 || pl.NTW != 2 || (pl.MTW != 1 && pl.MTW != 2) || (pl.KC != 16 && pl.KC != 32)) return false;
    // lane offsets into `in`, `out`, `r` and the partial tiles are 32-bit byte offsets
    const int64_t lim = (int64_t)1 << 32;
    if (((int64_t)g.n * in.sn + (int64_t)ci * in.sc) * 4 >= lim || ((int64_t)g.n * out.sn + (int64_t)co * out.sc) * 4 >= lim ||
        (r && ((int64_t)g.n * r->sn + (int64_t)co * r->sc) * 4 >= lim) || (int64_t)g.n * co * oh * ow * 4 >= lim)
        return false;
    C3Args a{};
    a.in = in.p; a.isn = in.sn; a.isc = in.sc;
    a.scale_shift = scale_shift;
    a.wq = wq; a.CIP = (ci + 7) / 8 * 8;
    a.r = r ? r->p : nullptr; a.rsn = r ? r->sn : 0; a.rsc = r ? r->sc : 0;
    a.out = out.p; a.osn = out.sn; a.osc = out.sc;
    a.N = g.n; a.H = g.h; a.W = g.w; a.CI = ci; a.CO = co; a.ep = (int)ep;
    a.stride = stride;
    a.TR = pl.TR; a.IMGS = pl.IMGS; a.bands = pl.bands;
    a.pix_per_img = pl.TR * ow; a.n_pix = pl.IMGS * pl.TR * ow;
    a.lrows = pl.lrows; a.lcols = pl.lcols; a.q_per_img = pl.q_per_img; a.in_items = pl.in_items;
    a.chunks = pl.chunks; a.cps = pl.cps;
    a.part = scratch; a.part_stride = (int64_t)g.n * co * oh * ow;
    const int ch = pl.WM * pl.MTW * 32;
    L.a = a;
    L.MTW = pl.MTW; L.KC = pl.KC; L.S = pl.S;
    // one staging item per thread at most: the variant whose activation loads run two chunks ahead
    L.NI = pl.in_items <= kThreads ? 1 : kInItems;
    L.a.wg_x = pl.bands * ((g.n + pl.IMGS - 1) / pl.IMGS);
    L.a.wg_x8 = (L.a.wg_x + 7) / 8 * 8;
    L.grid = dim3((unsigned)L.a.wg_x8, (unsigned)((co + ch - 1) / ch), (unsigned)pl.S);
    L.lds_bytes = pl.lds_bytes;
    L.scratch = scratch;
    return true;
}

void conv3x3_bf16_finish(Ctx &cx, const C3Launch &L, Geo g) {
    if (L.S <= 1) return;
    const C3Args &a = L.a;
    const int co = a.CO;
    const int64_t total = a.part_stride;
    // the values are final only here: this kernel leaves the statistics when its wavefronts are whole
    // runs of 64 pixels of one plane
    const int hw = g.h * g.w, rtiles = g.n * (hw / 64);
    const dim3 rgrid((unsigned)((total + kThreads - 1) / kThreads));
    // (a launch of its own in the accounts; the convolution's algorithmic bytes were counted with the first)
    const bool go = cx.launch(K_SPLITK_REDUCE, 0.0);
    if (cx.want_emit && cx.emit_buf && hw % 64 == 0 && total % kThreads == 0 &&
        (size_t)co * rtiles * 2 <= cx.emit_floats) {
        cx.emitted = EmittedStats{a.out, a.osn, a.osc, co, g.n, g.h, g.w, rtiles, 64};
        if (go)
            cx.run(splitk_reduce_k<true>, rgrid, dim3(kThreads), 0, L.scratch, a.part_stride, L.S, co, hw, total, a.r,
                   a.rsn, a.rsc, a.out, a.osn, a.osc, a.ep, cx.emit_buf, rtiles);
    } else if (go) {
        cx.run(splitk_reduce_k<false>, rgrid, dim3(kThreads), 0, L.scratch, a.part_stride, L.S, co, hw, total, a.r,
               a.rsn, a.rsc, a.out, a.osn, a.osc, a.ep, (float *)nullptr, 0);
    }
}

bool conv3x3_bf16(Ctx &cx, View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g,
                  Epilogue ep, const View *r, View out, float *scratch) {
    C3Launch L;
    if (!conv3x3_bf16_plan(in, scale_shift, wq, ci, co, g, ep, r, out, scratch, L)) return false;
    C3Args &a = L.a;
    // Statistics of the output for the BN layer that reads it next: no split (for split launches see
    // conv3x3_bf16_finish), and every pixel slot of every workgroup a valid pixel (whole blocks of rows or images).
    const int slots = 4 * 2 * 32, tiles = a.wg_x * 4;
    const bool whole = a.n_pix == slots && g.n % a.IMGS == 0 && g.h % a.TR == 0;
    if (cx.want_emit && cx.emit_buf && L.S == 1 && whole && (size_t)co * tiles * 2 <= cx.emit_floats) {
        a.emit = cx.emit_buf;
        a.emit_tiles = tiles;
        cx.emitted = EmittedStats{out.p, out.sn, out.sc, co, g.n, g.h, g.w, tiles, 64};
    }
    if (L.MTW == 1 && L.KC == 16) launch_c3<1, 1, 2, 16>(cx, L, L.grid);
    else if (L.MTW == 1 && L.KC == 32) launch_c3<1, 1, 2, 32>(cx, L, L.grid);
    else if (L.MTW == 2 && L.KC == 16) launch_c3<1, 2, 2, 16>(cx, L, L.grid);
    else launch_c3<1, 2, 2, 32>(cx, L, L.grid);
    conv3x3_bf16_finish(cx, L, g);
    return true;
}

// The same convolution with stride 2 (even h and w, zero padding 1): only the rows and columns of the
// result that exist are computed -- the pixel block of a workgroup is a block of the result, its input band
// twice as tall plus one row, and a result's operand records sit two rows and two columns apart.  `out`
// is [n][co][h/2][w/2]; no epilogue coupling, no epilogue statistics.
bool conv3x3_bf16_stride2(Ctx &cx, View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g, View out,
                          float *scratch) {
    C3Launch L;
    if (!conv3x3_bf16_plan(in, scale_shift, wq, ci, co, g, EP_STORE, nullptr, out, scratch, L, 2)) return false;
    const Geo low{g.n, g.h / 2, g.w / 2};
    const double P = (double)low.pixels();
    const double flops = 2.0 * P * ci * co * 9;
    cx.cost.conv_fwd_calls += 1;
    cx.cost.conv_flops += flops;
    cx.emitted = EmittedStats{};
    if (cx.launch(K_CONV_FWD, (double)g.pixels() * ci * 4.0 + P * co * 4.0, flops)) {
        if (L.MTW == 1 && L.KC == 16) launch_c3<1, 1, 2, 16>(cx, L, L.grid);
        else if (L.MTW == 1 && L.KC == 32) launch_c3<1, 1, 2, 32>(cx, L, L.grid);
        else if (L.MTW == 2 && L.KC == 16) launch_c3<1, 2, 2, 16>(cx, L, L.grid);
        else launch_c3<1, 2, 2, 32>(cx, L, L.grid);
    }
    conv3x3_bf16_finish(cx, L, low);
    return true;
}

}  // namespace rvn
