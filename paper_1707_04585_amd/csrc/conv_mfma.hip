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
#include "kernels.h"

namespace rvn {

namespace {

typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;

struct ConvArgs {
    const float *in;      // x (forward) or upstream gradient (data gradient)
    int64_t isn, isc;
    const float *scale_shift;  // [2*CI]: a = max(in*scale + shift, 0); null = use `in` as is
    const float *w;       // [CO][CI][KS][KS] forward; [CI][CO][KS][KS] read transposed+flipped otherwise
    const float *r;       // skip operand of the epilogue (may alias out)
    int64_t rsn, rsc;
    float *out;
    int64_t osn, osc;
    int N, H, W, CI, CO;
    int ep, transposed, round_bf16;
    int TH, IMGS, bands;          // rows per band, images per workgroup, bands per image
    int trows, tcols_log2, ctl;   // pixel tile shape (trows x tcols = 16), tiles per row
    int tiles_per_img, n_tiles;   // per workgroup
    int lrows, pitch, plane, img_stride;  // LDS geometry (floats)
    int tpr_log2;                 // threads per staged row
    float inv_lrows;
};

__device__ __forceinline__ float bf16_round_dev(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f;
    u += 0x7fffu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xffff0000u);
}

template <int KS, int MT, int NT, int KC>
__global__ __launch_bounds__(kThreads) void conv_mfma_f32_k(const ConvArgs p) {
    constexpr int KS2 = KS * KS, PAD = KS / 2, LP = KS == 3 ? 4 : 0;
    constexpr int WCHUNK = (KC / 4) * KS2 * MT * 64;  // filter floats per chunk
    extern __shared__ __align__(16) float smem[];
    float *in_lds = smem;
    float *w_lds = smem + p.IMGS * p.img_stride;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int band = blockIdx.x % p.bands, img_grp = blockIdx.x / p.bands;
    const int n0 = img_grp * p.IMGS;
    const int row0 = band * p.TH;
    const int co0 = blockIdx.y * (MT * 16);
    const int HW = p.H * p.W;

    // Per-tile LDS base address of this lane's pixel (B operand) and validity.
    const int tcols = 1 << p.tcols_log2;
    const int l16 = lane & 15, kq = lane >> 4;
    const int dr = l16 >> p.tcols_log2, dc = l16 & (tcols - 1);
    int b_base[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tile = wave + kWaves * t;
        const int img = tile / p.tiles_per_img, rem = tile - img * p.tiles_per_img;
        const int tr = rem / p.ctl, tc = rem - tr * p.ctl;
        b_base[t] = img * p.img_stride + kq * p.plane + (tr * p.trows + dr) * p.pitch + (LP - PAD) +
                    (tc << p.tcols_log2) + dc;
        if (tile >= p.n_tiles) b_base[t] = kq * p.plane;  // idle slot: any valid address
    }

    float4_t acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = float4_t{0.f, 0.f, 0.f, 0.f};

    const bool vec = (p.W & 3) == 0 && (p.isn & 3) == 0 && (p.isc & 3) == 0 &&
                     (reinterpret_cast<uintptr_t>(p.in) & 15) == 0;
    const int tpr = 1 << p.tpr_log2;
    const int tx = tid & (tpr - 1), ty = tid >> p.tpr_log2;
    const int rows_per_pass = kThreads >> p.tpr_log2;
    const int total_rows = p.IMGS * KC * p.lrows;

    // Right-hand zero quad of a staged row (3x3 only): the column just right of
    // the image must read as zero; it lies in the quad after the last data quad
    // unless W is not a multiple of 4 (then the masked tail of the data quad
    // covers it).
    const int quads = (p.W + 3) >> 2;
    const bool right_quad = KS == 3 && (p.W & 3) == 0;
    constexpr int RB = 6;                          // rows a thread loads before it stores
    constexpr int WITER = (WCHUNK + kThreads - 1) / kThreads;

    for (int c0 = 0; c0 < p.CI; c0 += KC) {
        __syncthreads();  // previous chunk fully consumed
        // ---- filter chunk: read global memory in its own order (runs of
        //      KC*KS2 floats per output channel, or MT*16*KS2 per input channel
        //      when transposed), all loads in flight before the first store.
        float wv[WITER];
        int wdst[WITER];
#pragma unroll
        for (int i = 0; i < WITER; ++i) {
            const int e = tid + i * kThreads;
            int kol, cl, t;
            if (p.transposed) {
                cl = e / (MT * 16 * KS2);
                const int rem = e - cl * (MT * 16 * KS2);
                kol = rem / KS2;
                t = rem - kol * KS2;
            } else {
                kol = e / (KC * KS2);
                const int rem = e - kol * (KC * KS2);
                cl = rem / KS2;
                t = rem - cl * KS2;
            }
            const int ko = co0 + kol, ch = c0 + cl;
            float v = 0.f;
            if (e < WCHUNK && ko < p.CO && ch < p.CI) {
                v = p.transposed ? p.w[((int64_t)ch * p.CO + ko) * KS2 + t]
                                 : p.w[((int64_t)ko * p.CI + ch) * KS2 + t];
            }
            wv[i] = v;
            // A-operand order; the transposed (data-gradient) filter is also flipped.
            const int tt = p.transposed ? KS2 - 1 - t : t;
            wdst[i] = e < WCHUNK ? ((((cl >> 2) * KS2 + tt) * MT + (kol >> 4)) * 64 + (cl & 3) * 16 + (kol & 15)) : -1;
        }
        // ---- input band: a = max(x*scale + shift, 0), zero outside the image
        for (int rbase = 0; rbase < total_rows; rbase += RB * rows_per_pass) {
            float4 q[RB];
            int dsti[RB];
            float sc[RB], sh[RB];
            bool live[RB];
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int rho = rbase + i * rows_per_pass + ty;
                const int pl = (int)(((float)rho + 0.5f) * p.inv_lrows);  // rho / lrows
                const int lr = rho - pl * p.lrows;
                const int img = pl / KC, c = pl - img * KC;
                const int n = n0 + img, ch = c0 + c, row = row0 - PAD + lr;
                const int col = tx * 4;
                dsti[i] = (rho < total_rows && tx < quads) ? img * p.img_stride + c * p.plane + lr * p.pitch + LP + col : -1;
                live[i] = dsti[i] >= 0 && n < p.N && ch < p.CI && row >= 0 && row < p.H;
                q[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                sc[i] = 1.f;
                sh[i] = 0.f;
                if (live[i]) {
                    const float *src = p.in + (int64_t)n * p.isn + (int64_t)ch * p.isc + row * p.W + col;
                    if (vec) {
                        q[i] = *reinterpret_cast<const float4 *>(src);
                    } else {
                        q[i].x = src[0];
                        if (col + 1 < p.W) q[i].y = src[1];
                        if (col + 2 < p.W) q[i].z = src[2];
                        if (col + 3 < p.W) q[i].w = src[3];
                    }
                    if (p.scale_shift) {
                        sc[i] = p.scale_shift[ch];
                        sh[i] = p.scale_shift[p.CI + ch];
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                if (dsti[i] < 0) continue;
                float v[4] = {q[i].x, q[i].y, q[i].z, q[i].w};
                if (live[i]) {
                    if (p.scale_shift) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] = fmaxf(fmaf(v[j], sc[i], sh[i]), 0.f);
                    }
                    if (p.round_bf16) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] = bf16_round_dev(v[j]);
                    }
                    if (!vec) {
                        const int col = tx * 4;
#pragma unroll
                        for (int j = 1; j < 4; ++j)
                            if (col + j >= p.W) v[j] = 0.f;
                    }
                }
                float *dst = in_lds + dsti[i];
                *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                if (KS == 3) {
                    if (tx == 0) *reinterpret_cast<float4 *>(dst - 4) = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (right_quad && tx == quads - 1)
                        *reinterpret_cast<float4 *>(dst + 4) = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < WITER; ++i) {
            if (wdst[i] >= 0) w_lds[wdst[i]] = p.round_bf16 ? bf16_round_dev(wv[i]) : wv[i];
        }
        __syncthreads();
        // ---- multiply
#pragma unroll
        for (int c4 = 0; c4 < KC / 4; ++c4) {
#pragma unroll
            for (int rr = 0; rr < KS; ++rr) {
#pragma unroll
                for (int ss = 0; ss < KS; ++ss) {
                    float a[MT];
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        a[m] = w_lds[((c4 * KS2 + rr * KS + ss) * MT + m) * 64 + lane];
                    const int off = c4 * 4 * p.plane + rr * p.pitch + ss;
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const float b = in_lds[b_base[t] + off];
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[m], b, acc[m][t], 0, 0, 0);
                    }
                }
            }
        }
    }

    // ---- epilogue: lane holds channels co0 + m*16 + 4*kq + j (j = 0..3) of its pixel.
    //      r may alias out (element for element), so the compiler cannot move a
    //      skip load above an earlier store: all skip values are requested first.
    int64_t e_off[NT];  // offset of (image, pixel) in out / r, -1: nothing to write
    int64_t e_roff[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tile = wave + kWaves * t;
        const int img = tile / p.tiles_per_img, rem = tile - img * p.tiles_per_img;
        const int tr = rem / p.ctl, tc = rem - tr * p.ctl;
        const int n = n0 + img, row = row0 + tr * p.trows + dr, col = (tc << p.tcols_log2) + dc;
        const bool ok = tile < p.n_tiles && n < p.N && row < p.H && row < row0 + p.TH && col < p.W;
        const int pix = row * p.W + col;
        e_off[t] = ok ? (int64_t)n * p.osn + pix : -1;
        e_roff[t] = (int64_t)n * p.rsn + pix;
    }
    if (p.ep != EP_STORE) {
        float rv[NT][MT][4];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ko = co0 + m * 16 + kq * 4 + j;
                    rv[t][m][j] = e_off[t] >= 0 && ko < p.CO ? p.r[e_roff[t] + (int64_t)ko * p.rsc] : 0.f;
                }
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[m][t][j] = p.ep == EP_ADD ? rv[t][m][j] + acc[m][t][j] : rv[t][m][j] - acc[m][t][j];
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (e_off[t] < 0) continue;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ko = co0 + m * 16 + kq * 4 + j;
                if (ko < p.CO) p.out[e_off[t] + (int64_t)ko * p.osc] = acc[m][t][j];
            }
        }
    }
    (void)HW;
}

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
    const int mt = co <= 16 ? 1 : co <= 32 ? 2 : 4;
    const int kc = ks == 3 ? (mt == 4 ? 8 : 16) : 16;
    const Tiling tl = choose_tiling(g, ks, kc, mt);
    if (tl.NT == 0) {  // no tiling fits (image rows too wide for LDS)
        cx.fail(hipErrorInvalidConfiguration);
        return;
    }
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
    a.tpr_log2 = ilog2((g.w + 3) / 4);
    a.inv_lrows = 1.0f / (float)a.lrows;
    dim3 grid((unsigned)(tl.bands * ((g.n + tl.IMGS - 1) / tl.IMGS)), (unsigned)((co + mt * 16 - 1) / (mt * 16)));
    if (ks == 3) {
        if (kc == 8) launch_conv<3, 8>(cx, a, tl, mt, grid);
        else launch_conv<3, 16>(cx, a, tl, mt, grid);
    } else {
        launch_conv<1, 16>(cx, a, tl, mt, grid);
    }
}

}  // namespace

void conv_fwd(Ctx &cx, View x, const float *scale_shift, rvn_dtype dt, const float *w, const uint16_t *wq, int cin,
              int cout, int ks, Geo g, Epilogue ep, const View *r, View out, float *scratch) {
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_fwd_calls += 1;
    cx.cost.conv_flops += flops;
    if (!cx.launch(K_CONV_FWD, P * cin * 4.0 + P * cout * 4.0 * (ep == EP_STORE ? 1.0 : 2.0), flops)) return;
    if (dt == RVN_BF16 && conv_bf16(cx, x, scale_shift, w, wq, false, cin, cout, ks, g, ep, r, out, scratch)) return;
    conv_mfma(cx, x, scale_shift, w, false, cin, cout, ks, g, dt == RVN_BF16, ep, r, out);
}

void conv_dgrad(Ctx &cx, View dh, rvn_dtype dt, const float *w, const uint16_t *wq, int cin, int cout, int ks,
                Geo g, float *da, float *scratch) {
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_dgrad_calls += 1;
    cx.cost.conv_flops += flops;
    if (!cx.launch(K_CONV_DGRAD, P * cout * 4.0 + P * cin * 4.0, flops)) return;
    // A stride-1 "same" convolution of dh (cout channels) with the transposed,
    // flipped filter, producing cin channels.
    if (dt == RVN_BF16 && conv_bf16(cx, dh, nullptr, w, wq, true, cout, cin, ks, g, EP_STORE, nullptr, dense_view(da, cin, g), scratch))
        return;
    conv_mfma(cx, dh, nullptr, w, true, cout, cin, ks, g, dt == RVN_BF16, EP_STORE, nullptr,
              dense_view(da, cin, g));
}

}  // namespace rvn
