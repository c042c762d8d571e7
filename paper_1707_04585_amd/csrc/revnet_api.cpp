// Host side of the library: argument validation, workspace planning and the
// block / stack drivers that sequence the HIP kernels.  Everything here runs
// on the host and only enqueues work on the caller's stream.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "kernels.h"

namespace rvn {
namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

struct Layer {
    int cin, cout, ks;
};

// Residual function shapes (Section 2.2): Basic = c3(c3(x)),
// Bottleneck = c1(c3(c1(x))) with the 1x1 convolutions reducing to `width`
// channels and projecting back.
int func_layers(const rvn_block_desc &d, Layer out[3]) {
    if (d.kind == RVN_BASIC) {
        out[0] = {d.c_half, d.c_half, 3};
        out[1] = {d.c_half, d.c_half, 3};
        return 2;
    }
    out[0] = {d.c_half, d.width, 1};
    out[1] = {d.width, d.width, 3};
    out[2] = {d.width, d.c_half, 1};
    return 3;
}

int check_desc(const rvn_block_desc *d) {
    if (!d) return fail(RVN_ERR_NULL, "descriptor is NULL");
    if (d->kind != RVN_BASIC && d->kind != RVN_BOTTLENECK)
        return fail(RVN_ERR_DTYPE, "unknown block kind %d", (int)d->kind);
    if (d->conv_dtype != RVN_F32 && d->conv_dtype != RVN_BF16)
        return fail(RVN_ERR_DTYPE, "unknown conv_dtype %d", (int)d->conv_dtype);
    if (d->c_half <= 0 || d->c_half > 65536)
        return fail(RVN_ERR_SHAPE, "c_half = %d out of range [1, 65536]", d->c_half);
    if (d->kind == RVN_BOTTLENECK && (d->width <= 0 || d->width > 65536))
        return fail(RVN_ERR_SHAPE, "bottleneck width = %d out of range [1, 65536]", d->width);
    if (!(d->bn_eps > 0.f)) return fail(RVN_ERR_SHAPE, "bn_eps must be > 0");
    return RVN_OK;
}

int check_geo(int64_t n, int64_t h, int64_t w) {
    if (n <= 0 || h <= 0 || w <= 0) return fail(RVN_ERR_SHAPE, "n, h, w must be positive (got %lld, %lld, %lld)", (long long)n, (long long)h, (long long)w);
    if (h > 32768 || w > 32768 || n > (1 << 24) || n * h * w > 0x7fffffffLL)
        return fail(RVN_ERR_SHAPE, "n*h*w = %lld exceeds the supported 2^31-1 pixels", (long long)(n * h * w));
    return RVN_OK;
}

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Workspace layout.  Offsets in bytes from the workspace base.
struct Plan {
    int L;
    Layer layers[3];
    size_t stats[3];      // kStatsArrays*cin floats each: mean, rstd, scale, shift
    size_t counters;      // ticket counters of the cross-workgroup reductions (ints)
    int n_counters;
    size_t bn_scratch;    // partial sums of the per-channel reductions
    size_t wgrad_scratch; // partial filter gradients (backward only)
    size_t conv_scratch;  // partial tiles of channel-split convolutions (kept apart: a filter gradient's
                          // partial results stay alive across the following data-gradient convolution)
    size_t h[2];          // h_l = conv_l(a_l), fp32, input of layer l+1
    size_t g[2];          // gradient ping-pong buffers (backward only)
    // bf16 convolutions with large filters: the filters of the function at hand
    // in bf16 and K order, for the forward convolution and (backward only) for
    // the data gradient; `prep[l]` says whether layer l uses them
    size_t wq_f[3], wq_b[3];
    bool prep[3];
    // fixed-point residual stream only: the function's input as fp32 and the
    // function's value before it is rounded into the stream
    size_t xf, fout;
    size_t total;
};

// Filters this large are converted once per function evaluation instead of in
// every workgroup of the convolution.
bool wants_prep(const rvn_block_desc &d, const Layer &ly, const Geo &g) {
    if (d.conv_dtype != RVN_BF16) return false;
    if (ly.ks == 1 && (conv1x1_direct_ok(ly.cin, g) || conv1x1_direct_ok(ly.cout, g))) return true;
    if (ly.ks == 3 && (conv3x3_bf16_ok(ly.cin, ly.cout, g) || conv3x3_bf16_ok(ly.cout, ly.cin, g))) return true;
    return (int64_t)ly.cin * ly.cout * ly.ks * ly.ks >= 16384;
}

Plan make_plan(const rvn_block_desc &d, const Geo &g, bool backward, bool fixed = false) {
    Plan p{};
    p.L = func_layers(d, p.layers);
    const size_t P = (size_t)g.pixels();
    size_t off = 0, bn_s = 0, wg_s = 0, cv_s = 0, max_cin = 0, max_mid = 0;
    for (int l = 0; l < p.L; ++l) {
        const Layer &ly = p.layers[l];
        p.stats[l] = off;
        off = align_up(off + kStatsArrays * (size_t)ly.cin * 4);
        bn_s = std::max(bn_s, bn_scratch_floats(ly.cin, g));
        if (backward) wg_s = std::max(wg_s, wgrad_scratch_floats(ly.cin, ly.cout, ly.ks, g));
        if (d.conv_dtype == RVN_BF16) {
            cv_s = std::max(cv_s, conv_bf16_scratch_floats(ly.cin, ly.cout, ly.ks, g));
            if (backward) cv_s = std::max(cv_s, conv_bf16_scratch_floats(ly.cout, ly.cin, ly.ks, g));
        }
        max_cin = std::max(max_cin, (size_t)ly.cin);
        if (l < p.L - 1) max_mid = std::max(max_mid, (size_t)ly.cout);
    }
    for (int l = 0; l < p.L; ++l) {
        const Layer &ly = p.layers[l];
        p.prep[l] = wants_prep(d, ly, g);
        if (!p.prep[l]) continue;
        p.wq_f[l] = off;
        off = align_up(off + filter_bf16_elems(ly.cout, ly.cin, ly.ks) * 2);
        if (backward) {
            p.wq_b[l] = off;
            off = align_up(off + filter_bf16_elems(ly.cin, ly.cout, ly.ks) * 2);
        }
    }
    p.counters = off;
    p.n_counters = (int)std::max(max_cin, (size_t)1) * kCounterStride;
    off = align_up(off + (size_t)p.n_counters * 4);
    p.bn_scratch = off;
    off = align_up(off + bn_s * 4);
    p.wgrad_scratch = off;
    off = align_up(off + wg_s * 4);
    p.conv_scratch = off;
    off = align_up(off + cv_s * 4);
    if (fixed) {
        p.xf = off;
        off = align_up(off + P * d.c_half * 4);
        p.fout = off;
        off = align_up(off + P * d.c_half * 4);
    }
    if (backward) {
        // a_l = ReLU(BN(x_l)) is never stored: every convolution kernel forms it
        // from x_l (the function input or h_{l-1}) while staging its operands.
        for (int l = 0; l < p.L - 1; ++l) {
            p.h[l] = off;
            off = align_up(off + P * p.layers[l].cout * 4);
        }
        for (int i = 0; i < 2; ++i) {
            p.g[i] = off;
            off = align_up(off + P * max_cin * 4);
        }
    } else {
        // Forward keeps nothing: a(x) is formed inside the convolution, and one
        // intermediate buffer is enough (h_l is dead once conv l+1 has run).
        const size_t h0 = off;
        off = align_up(off + P * max_mid * 4);
        const size_t h1 = off;
        if (p.L > 2) off = align_up(off + P * max_mid * 4);
        p.h[0] = h0;
        p.h[1] = p.L > 2 ? h1 : h0;
    }
    p.total = off;
    return p;
}

struct Bufs {
    float *stats[3];
    float *h[2];
    float *g[2];
    float *bn_scratch;
    float *wgrad_scratch, *conv_scratch;
    int *counters;
    uint16_t *wq_f[3], *wq_b[3];  // null where the layer does not use converted filters
    float *xf, *fout;
};

Bufs bind(const Plan &p, void *ws) {
    char *b = static_cast<char *>(ws);
    Bufs o{};
    for (int l = 0; l < 3; ++l) {
        o.stats[l] = reinterpret_cast<float *>(b + p.stats[l]);
        o.wq_f[l] = p.prep[l] ? reinterpret_cast<uint16_t *>(b + p.wq_f[l]) : nullptr;
        o.wq_b[l] = p.prep[l] && p.wq_b[l] ? reinterpret_cast<uint16_t *>(b + p.wq_b[l]) : nullptr;
    }
    for (int l = 0; l < 2; ++l) {
        o.h[l] = reinterpret_cast<float *>(b + p.h[l]);
        o.g[l] = reinterpret_cast<float *>(b + p.g[l]);
    }
    o.bn_scratch = reinterpret_cast<float *>(b + p.bn_scratch);
    o.counters = reinterpret_cast<int *>(b + p.counters);
    o.wgrad_scratch = reinterpret_cast<float *>(b + p.wgrad_scratch);
    o.conv_scratch = reinterpret_cast<float *>(b + p.conv_scratch);
    o.xf = reinterpret_cast<float *>(b + p.xf);
    o.fout = reinterpret_cast<float *>(b + p.fout);
    return o;
}

// ---- tensors ---------------------------------------------------------------

int check_tensor(const char *name, const rvn_tensor *t, const rvn_block_desc &d, const rvn_tensor *like) {
    if (!t) return fail(RVN_ERR_NULL, "tensor %s is NULL", name);
    if (!t->ptr) return fail(RVN_ERR_NULL, "tensor %s has a NULL data pointer", name);
    if (int rc = check_geo(t->n, t->h, t->w)) return rc;
    if (t->c != d.c_half)
        return fail(RVN_ERR_SHAPE, "tensor %s has c = %lld, descriptor says c_half = %d", name, (long long)t->c, d.c_half);
    if (like && (t->n != like->n || t->h != like->h || t->w != like->w))
        return fail(RVN_ERR_SHAPE, "tensor %s has shape [%lld,%lld,%lld,%lld], expected n,h,w = %lld,%lld,%lld", name,
                    (long long)t->n, (long long)t->c, (long long)t->h, (long long)t->w, (long long)like->n, (long long)like->h, (long long)like->w);
    const int64_t hw = t->h * t->w;
    if (t->sw != 1 || t->sh != t->w || t->sc < hw || t->sn < (t->c - 1) * t->sc + hw)
        return fail(RVN_ERR_STRIDE, "tensor %s: strides (%lld,%lld,%lld,%lld) unsupported; need sw=1, sh=w, sc>=h*w, sn>=(c-1)*sc+h*w",
                    name, (long long)t->sn, (long long)t->sc, (long long)t->sh, (long long)t->sw);
    if (reinterpret_cast<uintptr_t>(t->ptr) % 4)
        return fail(RVN_ERR_STRIDE, "tensor %s: data pointer is not 4-byte aligned", name);
    return RVN_OK;
}

bool same_tensor(const rvn_tensor *a, const rvn_tensor *b) {
    return a->ptr == b->ptr && a->sn == b->sn && a->sc == b->sc;
}

// Exact overlap test for two tensors of the supported layout: each occupies,
// per image, one interval of (c-1)*sc + h*w elements.
bool overlaps(const rvn_tensor *a, const rvn_tensor *b) {
    const int64_t la = ((a->c - 1) * a->sc + a->h * a->w) * 4, lb = ((b->c - 1) * b->sc + b->h * b->w) * 4;
    const int64_t pa = (int64_t)reinterpret_cast<uintptr_t>(a->ptr), pb = (int64_t)reinterpret_cast<uintptr_t>(b->ptr);
    const int64_t sa = a->sn * 4, sb = b->sn * 4;
    if (pa + (a->n - 1) * sa + la <= pb || pb + (b->n - 1) * sb + lb <= pa) return false;
    for (int64_t i = 0; i < a->n; ++i) {
        const int64_t s = pa + i * sa, e = s + la;
        // images m of b with pb + m*sb < e and pb + m*sb + lb > s
        int64_t m_lo = (s - pb - lb) / sb;  // candidates around the bounds
        for (int64_t m = std::max<int64_t>(0, m_lo - 1); m < b->n && pb + m * sb < e; ++m)
            if (pb + m * sb + lb > s) return true;
    }
    return false;
}

bool overlaps_range(const rvn_tensor *a, const void *p, size_t bytes) {
    const int64_t la = ((a->c - 1) * a->sc + a->h * a->w) * 4;
    const int64_t pa = (int64_t)reinterpret_cast<uintptr_t>(a->ptr), pb = (int64_t)reinterpret_cast<uintptr_t>(p);
    return !(pa + (a->n - 1) * a->sn * 4 + la <= pb || pb + (int64_t)bytes <= pa);
}

View view_of(const rvn_tensor *t) { return View{static_cast<float *>(t->ptr), t->sn, t->sc}; }

int check_params(const rvn_block_desc &d, const rvn_block_params *p, const char *what) {
    if (!p) return fail(RVN_ERR_NULL, "%s is NULL", what);
    Layer ly[3];
    const int L = func_layers(d, ly);
    const rvn_func_params *fs[2] = {&p->F, &p->G};
    for (int f = 0; f < 2; ++f)
        for (int l = 0; l < L; ++l)
            if (!fs[f]->conv_w[l] || !fs[f]->bn_gamma[l] || !fs[f]->bn_beta[l])
                return fail(RVN_ERR_NULL, "%s: %c layer %d has a NULL parameter pointer", what, f ? 'G' : 'F', l);
    return RVN_OK;
}

int check_grads(const rvn_block_desc &d, const rvn_block_grads *p, const char *what) {
    if (!p) return fail(RVN_ERR_NULL, "%s is NULL", what);
    Layer ly[3];
    const int L = func_layers(d, ly);
    const rvn_func_grads *fs[2] = {&p->F, &p->G};
    for (int f = 0; f < 2; ++f)
        for (int l = 0; l < L; ++l)
            if (!fs[f]->d_conv_w[l] || !fs[f]->d_bn_gamma[l] || !fs[f]->d_bn_beta[l])
                return fail(RVN_ERR_NULL, "%s: %c layer %d has a NULL gradient pointer", what, f ? 'G' : 'F', l);
    return RVN_OK;
}

int check_ws(const void *ws, size_t have, size_t need) {
    if (!ws) return fail(RVN_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", need);
    if (reinterpret_cast<uintptr_t>(ws) % kAlign) return fail(RVN_ERR_WORKSPACE, "workspace is not %zu-byte aligned", kAlign);
    if (have < need) return fail(RVN_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", have, need);
    return RVN_OK;
}

// ---- residual function drivers ----------------------------------------------

// out = ep(r, Func(x)); leaves the layer inputs h_l and the BN statistics in `b`.
// frac_bits > 0: x, r and out are fixed-point stream tensors (int32 codes of
// 2^-frac_bits).  The function then runs on the fp32 copy b.xf of x -- which
// func_backward reads as the function's input afterwards -- and its value is
// rounded into the stream by an integer add / subtract (Section 3.2,
// "Numerical error").
void func_forward(Ctx &cx, const rvn_block_desc &d, const Plan &pl, const Bufs &b, Geo g, View x,
                  const rvn_func_params &p, Epilogue ep, const View *r, View out, int frac_bits) {
    View cur = x;
    if (frac_bits) {
        fix_to_float(cx, x, pl.layers[0].cin, g, frac_bits, b.xf);
        cur = dense_view(b.xf, pl.layers[0].cin, g);
    }
    FilterPrep prep[3];
    for (int l = 0; l < pl.L; ++l)
        prep[l] = FilterPrep{p.conv_w[l], pl.layers[l].cin, pl.layers[l].cout, pl.layers[l].ks, b.wq_f[l], b.wq_b[l]};
    // The conversion rides in the first statistics launch of the function.
    double prep_bytes = 0.0;
    const PrepArgs pa = plan_filter_prep(prep, pl.L, g, &prep_bytes);
    for (int l = 0; l < pl.L; ++l) {
        const Layer &ly = pl.layers[l];
        bn_stats(cx, cur, ly.cin, g, d.bn_eps, p.bn_gamma[l], p.bn_beta[l], b.bn_scratch, b.counters, b.stats[l],
                 l == 0 && pa.jobs > 0 ? &pa : nullptr, l == 0 ? prep_bytes : 0.0);
        const float *scale_shift = b.stats[l] + 2 * ly.cin;
        if (l < pl.L - 1) {
            View h = dense_view(b.h[l], ly.cout, g);
            conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, EP_STORE, nullptr, h, b.conv_scratch);
            cur = h;
        } else if (frac_bits) {
            conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, EP_STORE, nullptr,
                     dense_view(b.fout, ly.cout, g), b.conv_scratch);
            fix_axpy(cx, *r, b.fout, ly.cout, g, frac_bits, ep == EP_SUB ? -1 : 1, out);
        } else {
            conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, ep, r, out, b.conv_scratch);
        }
    }
}

// Ordinary backprop through Func at the activations func_forward left in `b`
// (Section 2.1, the backprop rule): out = skip + (dFunc/dx)^T upstream, and
// the parameter gradients.
void func_backward(Ctx &cx, const rvn_block_desc &d, const Plan &pl, const Bufs &b, Geo g, View x,
                   const rvn_func_params &p, View upstream, const rvn_func_grads &gr, bool accumulate,
                   View skip, View out) {
    View dh = upstream;
    int cur = 0;
    for (int l = pl.L - 1; l >= 0; --l) {
        const Layer &ly = pl.layers[l];
        const View xl = l > 0 ? dense_view(b.h[l - 1], ly.cin, g) : x;
        // The ordered sum of the filter gradient's partial results rides in the
        // BN-backward apply launch below.
        WgradReduce red;
        float *da = b.g[cur];
        if (d.conv_dtype != RVN_F32 ||
            !conv_dgrad_wgrad_f32(cx, xl, b.stats[l] + 2 * ly.cin, dh, p.conv_w[l], ly.cin, ly.cout, ly.ks, g,
                                  b.wgrad_scratch, gr.d_conv_w[l], accumulate, da, &red)) {
            conv_wgrad(cx, xl, b.stats[l] + 2 * ly.cin, d.conv_dtype, dh, ly.cin, ly.cout, ly.ks, g, b.wgrad_scratch,
                       gr.d_conv_w[l], accumulate, &red);
            conv_dgrad(cx, dh, d.conv_dtype, p.conv_w[l], b.wq_b[l], ly.cin, ly.cout, ly.ks, g, da, b.conv_scratch);
        }
        if (l > 0) {
            View dx = dense_view(da, ly.cin, g);
            bn_relu_bwd(cx, xl, da, ly.cin, g, b.stats[l], b.bn_scratch, b.counters, gr.d_bn_gamma[l], gr.d_bn_beta[l],
                        accumulate, nullptr, dx, &red);
            dh = dx;
            cur ^= 1;
        } else {
            bn_relu_bwd(cx, x, da, ly.cin, g, b.stats[l], b.bn_scratch, b.counters, gr.d_bn_gamma[l], gr.d_bn_beta[l],
                        accumulate, &skip, out, &red);
        }
    }
}

// Section 3.1: y1 = x1 + F(x2); y2 = x2 + G(y1).
void block_forward(Ctx &cx, const rvn_block_desc &d, const Plan &pl, const Bufs &b, Geo g, View x1,
                   View x2, const rvn_block_params &p, View y1, View y2, int frac_bits) {
    func_forward(cx, d, pl, b, g, x2, p.F, EP_ADD, &x1, y1, frac_bits);
    func_forward(cx, d, pl, b, g, y1, p.G, EP_ADD, &x2, y2, frac_bits);
}

// Section 3.2, Algorithm 1, with G handled completely before F.  With a
// fixed-point stream (frac_bits > 0) the tensors y, x hold int32 codes and the
// derivatives stay fp32.
void block_backward(Ctx &cx, const rvn_block_desc &d, const Plan &pl, const Bufs &b, Geo g, View y1,
                    View y2, View dy1, View dy2, const rvn_block_params &p, View x1, View x2, View dx1,
                    View dx2, const rvn_block_grads &gr, bool accumulate, int frac_bits) {
    const View shadow = dense_view(b.xf, d.c_half, g);  // fp32 copy of the function input at hand
    // z1 = y1;  x2 = y2 - G(z1)
    func_forward(cx, d, pl, b, g, y1, p.G, EP_SUB, &y2, x2, frac_bits);
    // dz1 = dy1 + (dG/dz1)^T dy2;  dwG          (dx1 = dz1)
    func_backward(cx, d, pl, b, g, frac_bits ? shadow : y1, p.G, dy2, gr.G, accumulate, dy1, dx1);
    // x1 = z1 - F(x2)
    func_forward(cx, d, pl, b, g, x2, p.F, EP_SUB, &y1, x1, frac_bits);
    // dx2 = dy2 + (dF/dx2)^T dz1;  dwF
    func_backward(cx, d, pl, b, g, frac_bits ? shadow : x2, p.F, dx1, gr.F, accumulate, dy2, dx2);
}

int finish(Ctx &cx) {
    if (cx.err != hipSuccess) return fail(RVN_ERR_HIP, "HIP error: %s", hipGetErrorString(cx.err));
    return RVN_OK;
}

int check_fwd_args(const rvn_block_desc *desc, const rvn_tensor *x1, const rvn_tensor *x2,
                   const rvn_tensor *y1, const rvn_tensor *y2, void *ws, size_t ws_bytes, Plan *plan, Geo *geo,
                   bool fixed = false) {
    if (int rc = check_desc(desc)) return rc;
    if (int rc = check_tensor("x1", x1, *desc, nullptr)) return rc;
    if (int rc = check_tensor("x2", x2, *desc, x1)) return rc;
    if (int rc = check_tensor("y1", y1, *desc, x1)) return rc;
    if (int rc = check_tensor("y2", y2, *desc, x1)) return rc;
    const rvn_tensor *t[4] = {x1, x2, y1, y2};
    const char *nm[4] = {"x1", "x2", "y1", "y2"};
    for (int i = 0; i < 4; ++i)
        for (int j = i + 1; j < 4; ++j) {
            const bool allowed = (i == 0 && j == 2) || (i == 1 && j == 3);
            if (allowed && same_tensor(t[i], t[j])) continue;
            if (overlaps(t[i], t[j])) return fail(RVN_ERR_ALIAS, "%s and %s overlap", nm[i], nm[j]);
        }
    *geo = Geo{(int)x1->n, (int)x1->h, (int)x1->w};
    *plan = make_plan(*desc, *geo, false, fixed);
    if (int rc = check_ws(ws, ws_bytes, plan->total)) return rc;
    for (int i = 0; i < 4; ++i)
        if (overlaps_range(t[i], ws, plan->total)) return fail(RVN_ERR_ALIAS, "%s overlaps the workspace", nm[i]);
    return RVN_OK;
}

int check_bwd_args(const rvn_block_desc *desc, const rvn_tensor *y1, const rvn_tensor *y2,
                   const rvn_tensor *dy1, const rvn_tensor *dy2, const rvn_tensor *x1, const rvn_tensor *x2,
                   const rvn_tensor *dx1, const rvn_tensor *dx2, void *ws, size_t ws_bytes, Plan *plan, Geo *geo,
                   bool fixed = false) {
    if (int rc = check_desc(desc)) return rc;
    const rvn_tensor *t[8] = {y1, y2, dy1, dy2, x1, x2, dx1, dx2};
    const char *nm[8] = {"y1", "y2", "dy1", "dy2", "x1", "x2", "dx1", "dx2"};
    for (int i = 0; i < 8; ++i)
        if (int rc = check_tensor(nm[i], t[i], *desc, i ? y1 : nullptr)) return rc;
    for (int i = 0; i < 8; ++i)
        for (int j = i + 1; j < 8; ++j) {
            const bool allowed = j == i + 4;  // x_i with y_i, dx_i with dy_i
            if (allowed && same_tensor(t[i], t[j])) continue;
            if (overlaps(t[i], t[j])) return fail(RVN_ERR_ALIAS, "%s and %s overlap", nm[i], nm[j]);
        }
    *geo = Geo{(int)y1->n, (int)y1->h, (int)y1->w};
    *plan = make_plan(*desc, *geo, true, fixed);
    if (int rc = check_ws(ws, ws_bytes, plan->total)) return rc;
    for (int i = 0; i < 8; ++i)
        if (overlaps_range(t[i], ws, plan->total)) return fail(RVN_ERR_ALIAS, "%s overlaps the workspace", nm[i]);
    return RVN_OK;
}

void stack_forward(Ctx &cx, const rvn_block_desc &d, int depth, const Plan &pl, const Bufs &b, Geo g,
                   View x1, View x2, const rvn_block_params *params, View y1, View y2, int frac_bits = 0) {
    clear_counters(cx, b.counters, pl.n_counters);
    for (int k = 0; k < depth; ++k) {
        block_forward(cx, d, pl, b, g, k ? y1 : x1, k ? y2 : x2, params[k], y1, y2, frac_bits);
    }
}

void stack_backward(Ctx &cx, const rvn_block_desc &d, int depth, const Plan &pl, const Bufs &b, Geo g,
                    View y1, View y2, View dy1, View dy2, const rvn_block_params *params, View x1, View x2,
                    View dx1, View dx2, const rvn_block_grads *grads, bool accumulate, int frac_bits = 0) {
    clear_counters(cx, b.counters, pl.n_counters);
    for (int k = depth - 1; k >= 0; --k) {
        const bool top = k == depth - 1;
        block_backward(cx, d, pl, b, g, top ? y1 : x1, top ? y2 : x2, top ? dy1 : dx1, top ? dy2 : dx2,
                       params[k], x1, x2, dx1, dx2, grads[k], accumulate, frac_bits);
    }
}

// ---- non-reversible subsampling block --------------------------------------
//
// Section 3.1: reversible blocks have stride 1, so ordinary layers that change
// the resolution sit between the stages and have their inputs stored
// (Section 3.2).  The block built here (the paper leaves its form open):
//     a0 = ReLU(BN_0(x));  y = Conv_1x1,stride 2(a0; Ws) + R(x)
// with R the Basic / Bottleneck function with stride 2 on its 3x3 convolution.
// A stride-2 convolution runs as the stride-1 kernel followed by taking every
// second row and column (3x3), or on the subsampled input (1x1); its adjoints
// run as the stride-1 adjoints of the gradient spread out with zeros.

struct DownLayer {
    int cin, cout, ks;
    bool strided;
};

int down_layers(const rvn_down_desc &d, DownLayer out[3]) {
    if (d.kind == RVN_BASIC) {
        out[0] = {d.c_in, d.c_out, 3, true};
        out[1] = {d.c_out, d.c_out, 3, false};
        return 2;
    }
    out[0] = {d.c_in, d.width, 1, false};
    out[1] = {d.width, d.width, 3, true};
    out[2] = {d.width, d.c_out, 1, false};
    return 3;
}

int check_down_desc(const rvn_down_desc *d) {
    if (!d) return fail(RVN_ERR_NULL, "descriptor is NULL");
    if (d->kind != RVN_BASIC && d->kind != RVN_BOTTLENECK)
        return fail(RVN_ERR_DTYPE, "unknown block kind %d", (int)d->kind);
    if (d->conv_dtype != RVN_F32 && d->conv_dtype != RVN_BF16)
        return fail(RVN_ERR_DTYPE, "unknown conv_dtype %d", (int)d->conv_dtype);
    if (d->c_in <= 0 || d->c_in > 131072 || d->c_out <= 0 || d->c_out > 131072)
        return fail(RVN_ERR_SHAPE, "c_in = %d, c_out = %d out of range [1, 131072]", d->c_in, d->c_out);
    if (d->kind == RVN_BOTTLENECK && (d->width <= 0 || d->width > 65536))
        return fail(RVN_ERR_SHAPE, "bottleneck width = %d out of range [1, 65536]", d->width);
    if (!(d->bn_eps > 0.f)) return fail(RVN_ERR_SHAPE, "bn_eps must be > 0");
    return RVN_OK;
}

int check_down_geo(int64_t n, int64_t h, int64_t w) {
    if (int rc = check_geo(n, h, w)) return rc;
    if (h % 2 || w % 2) return fail(RVN_ERR_SHAPE, "h = %lld and w = %lld must be even", (long long)h, (long long)w);
    return RVN_OK;
}

constexpr int kShortcut = 3;  // slot of the shortcut's filter in the per-filter arrays

struct DownPlan {
    int L;
    DownLayer layers[3];
    Geo gin[3];  // geometry of layer l's input, which is that of the stride-1 convolution it runs
    Geo full, low;
    size_t stats[3];
    size_t counters;
    int n_counters;
    size_t bn_scratch, wgrad_scratch, conv_scratch;
    size_t wq_f[4], wq_b[4];  // bf16 filters (forward / data gradient); [kShortcut]: the shortcut
    bool bf16;
    size_t xs;     // x at the even positions, [n][c_in][h/2][w/2]
    size_t hfull;  // stride-1 result of the strided layer (forward); its gradient spread out (backward)
    size_t h[2];   // h_l, output of layer l < L-1 (subsampled for the strided one)
    size_t g[2];   // gradient ping-pong (backward only)
    size_t t;      // the shortcut's data gradient at half resolution (backward only)
    size_t total;
};

DownPlan make_down_plan(const rvn_down_desc &d, const Geo &full, bool backward) {
    DownPlan p{};
    p.L = down_layers(d, p.layers);
    p.full = full;
    p.low = Geo{full.n, full.h / 2, full.w / 2};
    p.bf16 = d.conv_dtype == RVN_BF16;
    bool below = false;
    size_t off = 0, bn_s = 0, wg_s = 0, cv_s = 0, max_cin = 0, max_g = 0;
    auto filt = [&](int slot, int cin, int cout, int ks, const Geo &g) {
        if (backward) wg_s = std::max(wg_s, wgrad_scratch_floats(cin, cout, ks, g));
        if (!p.bf16) return;
        cv_s = std::max(cv_s, conv_bf16_scratch_floats(cin, cout, ks, g));
        p.wq_f[slot] = off;
        off = align_up(off + filter_bf16_elems(cout, cin, ks) * 2);
        if (backward) {
            cv_s = std::max(cv_s, conv_bf16_scratch_floats(cout, cin, ks, g));
            p.wq_b[slot] = off;
            off = align_up(off + filter_bf16_elems(cin, cout, ks) * 2);
        }
    };
    for (int l = 0; l < p.L; ++l) {
        const DownLayer &ly = p.layers[l];
        p.gin[l] = below ? p.low : p.full;
        if (ly.strided) below = true;
        p.stats[l] = off;
        off = align_up(off + kStatsArrays * (size_t)ly.cin * 4);
        bn_s = std::max(bn_s, bn_scratch_floats(ly.cin, p.gin[l]));
        filt(l, ly.cin, ly.cout, ly.ks, p.gin[l]);
        max_cin = std::max(max_cin, (size_t)ly.cin);
        max_g = std::max(max_g, (size_t)p.gin[l].pixels() * ly.cin);
    }
    filt(kShortcut, d.c_in, d.c_out, 1, p.low);
    p.counters = off;
    p.n_counters = (int)max_cin * kCounterStride;
    off = align_up(off + (size_t)p.n_counters * 4);
    p.bn_scratch = off;
    off = align_up(off + bn_s * 4);
    p.wgrad_scratch = off;
    off = align_up(off + wg_s * 4);
    p.conv_scratch = off;
    off = align_up(off + cv_s * 4);
    p.xs = off;
    off = align_up(off + (size_t)p.low.pixels() * d.c_in * 4);
    for (int l = 0; l < p.L - 1; ++l) {
        const DownLayer &ly = p.layers[l];
        if (ly.strided) {
            p.hfull = off;
            off = align_up(off + (size_t)p.full.pixels() * ly.cout * 4);
        }
        p.h[l] = off;  // geometry of the next layer's input
        off = align_up(off + (size_t)p.gin[l + 1].pixels() * ly.cout * 4);
    }
    if (backward) {
        for (int i = 0; i < 2; ++i) {
            p.g[i] = off;
            off = align_up(off + max_g * 4);
        }
        p.t = off;
        off = align_up(off + (size_t)p.low.pixels() * d.c_in * 4);
    }
    p.total = off;
    return p;
}

struct DownBufs {
    float *stats[3], *h[2], *g[2];
    float *bn_scratch, *wgrad_scratch, *conv_scratch, *xs, *hfull, *t;
    int *counters;
    uint16_t *wq_f[4], *wq_b[4];
};

DownBufs bind(const DownPlan &p, void *ws, bool backward) {
    char *b = static_cast<char *>(ws);
    auto f = [&](size_t off) { return reinterpret_cast<float *>(b + off); };
    DownBufs o{};
    for (int l = 0; l < 3; ++l) o.stats[l] = f(p.stats[l]);
    for (int l = 0; l < 4; ++l) {
        o.wq_f[l] = p.bf16 ? reinterpret_cast<uint16_t *>(b + p.wq_f[l]) : nullptr;
        o.wq_b[l] = p.bf16 && backward ? reinterpret_cast<uint16_t *>(b + p.wq_b[l]) : nullptr;
    }
    for (int l = 0; l < 2; ++l) {
        o.h[l] = f(p.h[l]);
        o.g[l] = f(p.g[l]);
    }
    o.bn_scratch = f(p.bn_scratch);
    o.wgrad_scratch = f(p.wgrad_scratch);
    o.conv_scratch = f(p.conv_scratch);
    o.xs = f(p.xs);
    o.hfull = f(p.hfull);
    o.t = f(p.t);
    o.counters = reinterpret_cast<int *>(b + p.counters);
    return o;
}

// One filter to bf16, in the order the convolutions at geometry g read it.
void prep_one(Ctx &cx, const float *w, int cin, int cout, int ks, const Geo &g, uint16_t *qf, uint16_t *qb) {
    if (!qf && !qb) return;
    const FilterPrep fp{w, cin, cout, ks, qf, qb};
    double bytes = 0.0;
    const PrepArgs pa = plan_filter_prep(&fp, 1, g, &bytes);
    prep_filters_bf16(cx, pa, bytes);
}

// With recompute_only the internals (statistics, h_l, subsampled x) are left
// in `b` for down_backward and y is not formed.
void down_forward(Ctx &cx, const rvn_down_desc &d, const DownPlan &pl, const DownBufs &b, View x,
                  const rvn_down_params &p, View y, bool recompute_only) {
    clear_counters(cx, b.counters, pl.n_counters);
    for (int l = 0; l < pl.L; ++l)
        prep_one(cx, p.R.conv_w[l], pl.layers[l].cin, pl.layers[l].cout, pl.layers[l].ks, pl.gin[l], b.wq_f[l], b.wq_b[l]);
    prep_one(cx, p.shortcut_w, d.c_in, d.c_out, 1, pl.low, b.wq_f[kShortcut], b.wq_b[kShortcut]);
    View cur = x;
    for (int l = 0; l < pl.L; ++l) {
        const DownLayer &ly = pl.layers[l];
        const Geo g = pl.gin[l];
        bn_stats(cx, cur, ly.cin, g, d.bn_eps, p.R.bn_gamma[l], p.R.bn_beta[l], b.bn_scratch, b.counters, b.stats[l]);
        const float *scale_shift = b.stats[l] + 2 * ly.cin;
        if (l == 0) {
            // shortcut: the 1x1 stride-2 convolution of a0 is the 1x1 convolution of
            // a0 at the even positions, and a0 there needs only x there
            subsample2(cx, x, d.c_in, pl.full, b.xs);
            if (!recompute_only)
                conv_fwd(cx, dense_view(b.xs, d.c_in, pl.low), scale_shift, d.conv_dtype, p.shortcut_w, b.wq_f[kShortcut],
                         d.c_in, d.c_out, 1, pl.low, EP_STORE, nullptr, y, b.conv_scratch);
        }
        if (l == pl.L - 1) {
            if (!recompute_only)
                conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.R.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, EP_ADD, &y,
                         y, b.conv_scratch);
        } else if (ly.strided) {
            const View hf = dense_view(b.hfull, ly.cout, pl.full);
            conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.R.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, EP_STORE,
                     nullptr, hf, b.conv_scratch);
            subsample2(cx, hf, ly.cout, pl.full, b.h[l]);
            cur = dense_view(b.h[l], ly.cout, pl.low);
        } else {
            const View h = dense_view(b.h[l], ly.cout, g);
            conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.R.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, EP_STORE,
                     nullptr, h, b.conv_scratch);
            cur = h;
        }
    }
}

// Ordinary backprop (Section 2.1) from the stored input x.
void down_backward(Ctx &cx, const rvn_down_desc &d, const DownPlan &pl, const DownBufs &b, View x, View dy,
                   const rvn_down_params &p, View dx, const rvn_down_grads &gr, bool accumulate) {
    down_forward(cx, d, pl, b, x, p, View{}, true);
    View dcur = dy;
    int cur = 0;
    for (int l = pl.L - 1; l >= 0; --l) {
        const DownLayer &ly = pl.layers[l];
        const Geo g = pl.gin[l];
        const View xl = l > 0 ? dense_view(b.h[l - 1], ly.cin, g) : x;
        const float *scale_shift = b.stats[l] + 2 * ly.cin;
        if (ly.strided) {  // the upstream gradient here is dense: it left a BN backward below
            upsample2_zero(cx, dcur.p, ly.cout, pl.full, b.hfull);
            dcur = dense_view(b.hfull, ly.cout, pl.full);
        }
        float *da = b.g[cur];
        if (l == 0) {
            // a0's second child, the shortcut; first, because its filter gradient's
            // partial sums share the scratch with those of this layer, which stay
            // pending until the BN backward below
            conv_wgrad(cx, dense_view(b.xs, d.c_in, pl.low), scale_shift, d.conv_dtype, dy, d.c_in, d.c_out, 1, pl.low,
                       b.wgrad_scratch, gr.d_shortcut_w, accumulate);
            conv_dgrad(cx, dy, d.conv_dtype, p.shortcut_w, b.wq_b[kShortcut], d.c_in, d.c_out, 1, pl.low, b.t, b.conv_scratch);
        }
        WgradReduce red;
        conv_wgrad(cx, xl, scale_shift, d.conv_dtype, dcur, ly.cin, ly.cout, ly.ks, g, b.wgrad_scratch, gr.R.d_conv_w[l],
                   accumulate, &red);
        conv_dgrad(cx, dcur, d.conv_dtype, p.R.conv_w[l], b.wq_b[l], ly.cin, ly.cout, ly.ks, g, da, b.conv_scratch);
        if (l == 0) upsample2_add(cx, b.t, d.c_in, pl.full, da);
        const View out = l == 0 ? dx : dense_view(da, ly.cin, g);
        bn_relu_bwd(cx, xl, da, ly.cin, g, b.stats[l], b.bn_scratch, b.counters, gr.R.d_bn_gamma[l], gr.R.d_bn_beta[l],
                    accumulate, nullptr, out, &red);
        dcur = out;
        cur ^= 1;
    }
}

int check_any_tensor(const char *name, const rvn_tensor *t, int64_t c, int64_t n, int64_t h, int64_t w) {
    if (!t) return fail(RVN_ERR_NULL, "tensor %s is NULL", name);
    if (!t->ptr) return fail(RVN_ERR_NULL, "tensor %s has a NULL data pointer", name);
    if (t->n != n || t->c != c || t->h != h || t->w != w)
        return fail(RVN_ERR_SHAPE, "tensor %s has shape [%lld,%lld,%lld,%lld], expected [%lld,%lld,%lld,%lld]", name,
                    (long long)t->n, (long long)t->c, (long long)t->h, (long long)t->w, (long long)n, (long long)c,
                    (long long)h, (long long)w);
    const int64_t hw = h * w;
    if (t->sw != 1 || t->sh != w || t->sc < hw || t->sn < (c - 1) * t->sc + hw)
        return fail(RVN_ERR_STRIDE, "tensor %s: strides (%lld,%lld,%lld,%lld) unsupported; need sw=1, sh=w, sc>=h*w, sn>=(c-1)*sc+h*w",
                    name, (long long)t->sn, (long long)t->sc, (long long)t->sh, (long long)t->sw);
    if (reinterpret_cast<uintptr_t>(t->ptr) % 4)
        return fail(RVN_ERR_STRIDE, "tensor %s: data pointer is not 4-byte aligned", name);
    return RVN_OK;
}

int check_down_params(const rvn_down_desc &d, const rvn_down_params *p) {
    if (!p) return fail(RVN_ERR_NULL, "params is NULL");
    DownLayer ly[3];
    const int L = down_layers(d, ly);
    for (int l = 0; l < L; ++l)
        if (!p->R.conv_w[l] || !p->R.bn_gamma[l] || !p->R.bn_beta[l])
            return fail(RVN_ERR_NULL, "params: layer %d has a NULL parameter pointer", l);
    if (!p->shortcut_w) return fail(RVN_ERR_NULL, "params: shortcut_w is NULL");
    return RVN_OK;
}

int check_down_grads(const rvn_down_desc &d, const rvn_down_grads *p) {
    if (!p) return fail(RVN_ERR_NULL, "grads is NULL");
    DownLayer ly[3];
    const int L = down_layers(d, ly);
    for (int l = 0; l < L; ++l)
        if (!p->R.d_conv_w[l] || !p->R.d_bn_gamma[l] || !p->R.d_bn_beta[l])
            return fail(RVN_ERR_NULL, "grads: layer %d has a NULL gradient pointer", l);
    if (!p->d_shortcut_w) return fail(RVN_ERR_NULL, "grads: d_shortcut_w is NULL");
    return RVN_OK;
}

// ---- body: reversible stages joined by subsampling blocks -------------------

int check_body_desc(const rvn_body_desc *bd, int64_t n, int64_t h, int64_t w) {
    if (!bd) return fail(RVN_ERR_NULL, "descriptor is NULL");
    if (bd->stages < 1 || bd->stages > RVN_MAX_STAGES)
        return fail(RVN_ERR_SHAPE, "stages = %d out of range [1, %d]", bd->stages, RVN_MAX_STAGES);
    for (int s = 0; s < bd->stages; ++s) {
        if (int rc = check_desc(&bd->stage[s])) return rc;
        if (bd->depth[s] <= 0) return fail(RVN_ERR_SHAPE, "depth[%d] = %d must be positive", s, bd->depth[s]);
        if (s + 1 < bd->stages) {
            if (int rc = check_down_desc(&bd->down[s])) return rc;
            if (bd->down[s].c_in != 2 * bd->stage[s].c_half || bd->down[s].c_out != 2 * bd->stage[s + 1].c_half)
                return fail(RVN_ERR_SHAPE, "down[%d] maps %d -> %d channels, the stages have %d and %d", s, bd->down[s].c_in,
                            bd->down[s].c_out, 2 * bd->stage[s].c_half, 2 * bd->stage[s + 1].c_half);
            if (int rc = check_down_geo(n, h >> s, w >> s)) return rc;
        } else if (int rc = check_geo(n, h >> s, w >> s)) {
            return rc;
        }
    }
    return RVN_OK;
}

size_t body_ws_bytes(const rvn_body_desc &bd, const Geo &g0, bool backward) {
    size_t need = 0;
    for (int s = 0; s < bd.stages; ++s) {
        const Geo g{g0.n, g0.h >> s, g0.w >> s};
        need = std::max(need, make_plan(bd.stage[s], g, backward).total);
        if (s + 1 < bd.stages) need = std::max(need, make_down_plan(bd.down[s], g, backward).total);
    }
    return need;
}

View half_view(const rvn_tensor *t, int which) {
    return View{static_cast<float *>(t->ptr) + (int64_t)which * (t->c / 2) * t->sc, t->sn, t->sc};
}

}  // namespace
}  // namespace rvn

using namespace rvn;

extern "C" {

int revnet_version(void) { return 1000; }

const char *revnet_last_error(void) { return g_err; }

int revnet_workspace_bytes(const rvn_block_desc *desc, int64_t n, int64_t h, int64_t w,
                           size_t *fwd_bytes, size_t *bwd_bytes) {
    if (int rc = check_desc(desc)) return rc;
    if (int rc = check_geo(n, h, w)) return rc;
    const Geo g{(int)n, (int)h, (int)w};
    if (fwd_bytes) *fwd_bytes = make_plan(*desc, g, false).total;
    if (bwd_bytes) *bwd_bytes = make_plan(*desc, g, true).total;
    return RVN_OK;
}

int revnet_block_fwd(const rvn_block_desc *desc, const rvn_tensor *x1, const rvn_tensor *x2,
                     const rvn_block_params *params, const rvn_tensor *y1, const rvn_tensor *y2,
                     void *ws, size_t ws_bytes, void *hip_stream) {
    return revnet_stack_fwd(desc, 1, x1, x2, params, y1, y2, ws, ws_bytes, hip_stream);
}

int revnet_stack_fwd(const rvn_block_desc *desc, int32_t depth, const rvn_tensor *x1,
                     const rvn_tensor *x2, const rvn_block_params *params, const rvn_tensor *y1,
                     const rvn_tensor *y2, void *ws, size_t ws_bytes, void *hip_stream) {
    Plan pl;
    Geo g;
    if (depth <= 0) return fail(RVN_ERR_SHAPE, "depth = %d must be positive", depth);
    if (int rc = check_fwd_args(desc, x1, x2, y1, y2, ws, ws_bytes, &pl, &g)) return rc;
    if (!params) return fail(RVN_ERR_NULL, "params is NULL");
    for (int k = 0; k < depth; ++k)
        if (int rc = check_params(*desc, &params[k], "params")) return rc;
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    stack_forward(cx, *desc, depth, pl, bind(pl, ws), g, view_of(x1), view_of(x2), params, view_of(y1), view_of(y2));
    return finish(cx);
}

int revnet_block_bwd_reconstruct(const rvn_block_desc *desc, const rvn_tensor *y1, const rvn_tensor *y2,
                                 const rvn_tensor *dy1, const rvn_tensor *dy2,
                                 const rvn_block_params *params, const rvn_tensor *x1,
                                 const rvn_tensor *x2, const rvn_tensor *dx1, const rvn_tensor *dx2,
                                 const rvn_block_grads *grads, int accumulate_wgrads, void *ws,
                                 size_t ws_bytes, void *hip_stream) {
    return revnet_stack_bwd(desc, 1, y1, y2, dy1, dy2, params, x1, x2, dx1, dx2, grads, accumulate_wgrads,
                            ws, ws_bytes, hip_stream);
}

int revnet_stack_bwd(const rvn_block_desc *desc, int32_t depth, const rvn_tensor *y1,
                     const rvn_tensor *y2, const rvn_tensor *dy1, const rvn_tensor *dy2,
                     const rvn_block_params *params, const rvn_tensor *x1, const rvn_tensor *x2,
                     const rvn_tensor *dx1, const rvn_tensor *dx2, const rvn_block_grads *grads,
                     int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream) {
    Plan pl;
    Geo g;
    if (depth <= 0) return fail(RVN_ERR_SHAPE, "depth = %d must be positive", depth);
    if (int rc = check_bwd_args(desc, y1, y2, dy1, dy2, x1, x2, dx1, dx2, ws, ws_bytes, &pl, &g)) return rc;
    if (!params) return fail(RVN_ERR_NULL, "params is NULL");
    if (!grads) return fail(RVN_ERR_NULL, "grads is NULL");
    for (int k = 0; k < depth; ++k) {
        if (int rc = check_params(*desc, &params[k], "params")) return rc;
        if (int rc = check_grads(*desc, &grads[k], "grads")) return rc;
    }
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    stack_backward(cx, *desc, depth, pl, bind(pl, ws), g, view_of(y1), view_of(y2), view_of(dy1), view_of(dy2),
                   params, view_of(x1), view_of(x2), view_of(dx1), view_of(dx2), grads, accumulate_wgrads != 0);
    return finish(cx);
}

int revnet_stack_cost(const rvn_block_desc *desc, int32_t depth, int64_t n, int64_t h, int64_t w,
                      rvn_cost *fwd, rvn_cost *bwd) {
    if (int rc = check_desc(desc)) return rc;
    if (int rc = check_geo(n, h, w)) return rc;
    if (depth <= 0) return fail(RVN_ERR_SHAPE, "depth = %d must be positive", depth);
    const Geo g{(int)n, (int)h, (int)w};
    // Run the real drivers in counting mode on placeholder addresses; nothing
    // is dereferenced and nothing is launched.
    std::vector<rvn_block_params> params((size_t)depth);
    std::vector<rvn_block_grads> grads((size_t)depth);
    std::memset(params.data(), 0, params.size() * sizeof(rvn_block_params));
    std::memset(grads.data(), 0, grads.size() * sizeof(rvn_block_grads));
    const View v = dense_view(nullptr, desc->c_half, g);
    if (fwd) {
        const Plan pl = make_plan(*desc, g, false);
        Ctx cx;
        cx.dry = true;
        stack_forward(cx, *desc, depth, pl, bind(pl, nullptr), g, v, v, params.data(), v, v);
        *fwd = cx.cost;
    }
    if (bwd) {
        const Plan pl = make_plan(*desc, g, true);
        Ctx cx;
        cx.dry = true;
        stack_backward(cx, *desc, depth, pl, bind(pl, nullptr), g, v, v, v, v, params.data(), v, v, v, v,
                       grads.data(), false);
        *bwd = cx.cost;
    }
    return RVN_OK;
}

int revnet_down_workspace_bytes(const rvn_down_desc *desc, int64_t n, int64_t h, int64_t w, size_t *fwd_bytes,
                                size_t *bwd_bytes) {
    if (int rc = check_down_desc(desc)) return rc;
    if (int rc = check_down_geo(n, h, w)) return rc;
    const Geo g{(int)n, (int)h, (int)w};
    if (fwd_bytes) *fwd_bytes = make_down_plan(*desc, g, false).total;
    if (bwd_bytes) *bwd_bytes = make_down_plan(*desc, g, true).total;
    return RVN_OK;
}

int revnet_down_fwd(const rvn_down_desc *desc, const rvn_tensor *x, const rvn_down_params *params,
                    const rvn_tensor *y, void *ws, size_t ws_bytes, void *hip_stream) {
    if (int rc = check_down_desc(desc)) return rc;
    if (!x) return fail(RVN_ERR_NULL, "tensor x is NULL");
    if (int rc = check_down_geo(x->n, x->h, x->w)) return rc;
    if (int rc = check_any_tensor("x", x, desc->c_in, x->n, x->h, x->w)) return rc;
    if (int rc = check_any_tensor("y", y, desc->c_out, x->n, x->h / 2, x->w / 2)) return rc;
    if (int rc = check_down_params(*desc, params)) return rc;
    if (overlaps(x, y)) return fail(RVN_ERR_ALIAS, "x and y overlap");
    const Geo g{(int)x->n, (int)x->h, (int)x->w};
    const DownPlan pl = make_down_plan(*desc, g, false);
    if (int rc = check_ws(ws, ws_bytes, pl.total)) return rc;
    if (overlaps_range(x, ws, pl.total) || overlaps_range(y, ws, pl.total))
        return fail(RVN_ERR_ALIAS, "a tensor overlaps the workspace");
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    down_forward(cx, *desc, pl, bind(pl, ws, false), view_of(x), *params, view_of(y), false);
    return finish(cx);
}

int revnet_down_bwd(const rvn_down_desc *desc, const rvn_tensor *x, const rvn_tensor *dy,
                    const rvn_down_params *params, const rvn_tensor *dx, const rvn_down_grads *grads,
                    int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream) {
    if (int rc = check_down_desc(desc)) return rc;
    if (!x) return fail(RVN_ERR_NULL, "tensor x is NULL");
    if (int rc = check_down_geo(x->n, x->h, x->w)) return rc;
    if (int rc = check_any_tensor("x", x, desc->c_in, x->n, x->h, x->w)) return rc;
    if (int rc = check_any_tensor("dy", dy, desc->c_out, x->n, x->h / 2, x->w / 2)) return rc;
    if (int rc = check_any_tensor("dx", dx, desc->c_in, x->n, x->h, x->w)) return rc;
    if (int rc = check_down_params(*desc, params)) return rc;
    if (int rc = check_down_grads(*desc, grads)) return rc;
    if (overlaps(x, dy) || overlaps(x, dx) || overlaps(dy, dx)) return fail(RVN_ERR_ALIAS, "x, dy and dx must not overlap");
    const Geo g{(int)x->n, (int)x->h, (int)x->w};
    const DownPlan pl = make_down_plan(*desc, g, true);
    if (int rc = check_ws(ws, ws_bytes, pl.total)) return rc;
    if (overlaps_range(x, ws, pl.total) || overlaps_range(dy, ws, pl.total) || overlaps_range(dx, ws, pl.total))
        return fail(RVN_ERR_ALIAS, "a tensor overlaps the workspace");
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    down_backward(cx, *desc, pl, bind(pl, ws, true), view_of(x), view_of(dy), *params, view_of(dx), *grads,
                  accumulate_wgrads != 0);
    return finish(cx);
}

int revnet_body_workspace_bytes(const rvn_body_desc *desc, int64_t n, int64_t h, int64_t w, size_t *fwd_bytes,
                                size_t *bwd_bytes) {
    if (int rc = check_body_desc(desc, n, h, w)) return rc;
    const Geo g{(int)n, (int)h, (int)w};
    if (fwd_bytes) *fwd_bytes = body_ws_bytes(*desc, g, false);
    if (bwd_bytes) *bwd_bytes = body_ws_bytes(*desc, g, true);
    return RVN_OK;
}

namespace {

// Shapes, strides and overlaps of the per-stage tensors of a body call.
int check_body_tensors(const rvn_body_desc &bd, const char *name, const rvn_tensor *t, int64_t n, int64_t h, int64_t w) {
    if (!t) return fail(RVN_ERR_NULL, "%s is NULL", name);
    for (int s = 0; s < bd.stages; ++s) {
        char nm[32];
        snprintf(nm, sizeof nm, "%s[%d]", name, s);
        if (int rc = check_any_tensor(nm, &t[s], 2 * (int64_t)bd.stage[s].c_half, n, h >> s, w >> s)) return rc;
        for (int r = 0; r < s; ++r)
            if (overlaps(&t[r], &t[s])) return fail(RVN_ERR_ALIAS, "%s[%d] and %s[%d] overlap", name, r, name, s);
    }
    return RVN_OK;
}

}  // namespace

int revnet_body_fwd(const rvn_body_desc *desc, const rvn_tensor *x, const rvn_block_params *const *stage_params,
                    const rvn_down_params *down_params, const rvn_tensor *tops, void *ws, size_t ws_bytes,
                    void *hip_stream) {
    if (!x) return fail(RVN_ERR_NULL, "tensor x is NULL");
    if (int rc = check_body_desc(desc, x->n, x->h, x->w)) return rc;
    const rvn_body_desc &bd = *desc;
    if (int rc = check_any_tensor("x", x, 2 * (int64_t)bd.stage[0].c_half, x->n, x->h, x->w)) return rc;
    if (int rc = check_body_tensors(bd, "tops", tops, x->n, x->h, x->w)) return rc;
    if (!stage_params) return fail(RVN_ERR_NULL, "stage_params is NULL");
    if (bd.stages > 1 && !down_params) return fail(RVN_ERR_NULL, "down_params is NULL");
    for (int s = 0; s < bd.stages; ++s) {
        if (!stage_params[s]) return fail(RVN_ERR_NULL, "stage_params[%d] is NULL", s);
        for (int k = 0; k < bd.depth[s]; ++k)
            if (int rc = check_params(bd.stage[s], &stage_params[s][k], "stage_params")) return rc;
        if (s + 1 < bd.stages)
            if (int rc = check_down_params(bd.down[s], &down_params[s])) return rc;
        const bool same = s == 0 && same_tensor(x, &tops[0]);
        if (!same && overlaps(x, &tops[s])) return fail(RVN_ERR_ALIAS, "x and tops[%d] overlap", s);
    }
    const Geo g0{(int)x->n, (int)x->h, (int)x->w};
    const size_t need = body_ws_bytes(bd, g0, false);
    if (int rc = check_ws(ws, ws_bytes, need)) return rc;
    if (overlaps_range(x, ws, need)) return fail(RVN_ERR_ALIAS, "x overlaps the workspace");
    for (int s = 0; s < bd.stages; ++s)
        if (overlaps_range(&tops[s], ws, need)) return fail(RVN_ERR_ALIAS, "tops[%d] overlaps the workspace", s);
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    for (int s = 0; s < bd.stages; ++s) {
        const Geo g{g0.n, g0.h >> s, g0.w >> s};
        const Plan pl = make_plan(bd.stage[s], g, false);
        const rvn_tensor *in = s == 0 ? x : &tops[s];  // later stages run in place on the subsampling block's output
        stack_forward(cx, bd.stage[s], bd.depth[s], pl, bind(pl, ws), g, half_view(in, 0), half_view(in, 1),
                      stage_params[s], half_view(&tops[s], 0), half_view(&tops[s], 1));
        if (s + 1 < bd.stages) {
            const DownPlan dp = make_down_plan(bd.down[s], g, false);
            down_forward(cx, bd.down[s], dp, bind(dp, ws, false), view_of(&tops[s]), down_params[s], view_of(&tops[s + 1]),
                         false);
        }
    }
    return finish(cx);
}

int revnet_body_bwd(const rvn_body_desc *desc, const rvn_tensor *tops, const rvn_tensor *dtops,
                    const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                    const rvn_block_grads *const *stage_grads, const rvn_down_grads *down_grads,
                    int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!tops) return fail(RVN_ERR_NULL, "tops is NULL");
    if (int rc = check_body_desc(desc, tops[0].n, tops[0].h, tops[0].w)) return rc;
    const rvn_body_desc &bd = *desc;
    const int64_t n = tops[0].n, h = tops[0].h, w = tops[0].w;
    if (int rc = check_body_tensors(bd, "tops", tops, n, h, w)) return rc;
    if (int rc = check_body_tensors(bd, "dtops", dtops, n, h, w)) return rc;
    if (!stage_params || !stage_grads) return fail(RVN_ERR_NULL, "stage_params or stage_grads is NULL");
    if (bd.stages > 1 && (!down_params || !down_grads)) return fail(RVN_ERR_NULL, "down_params or down_grads is NULL");
    for (int s = 0; s < bd.stages; ++s) {
        if (!stage_params[s] || !stage_grads[s]) return fail(RVN_ERR_NULL, "stage_params[%d] or stage_grads[%d] is NULL", s, s);
        for (int k = 0; k < bd.depth[s]; ++k) {
            if (int rc = check_params(bd.stage[s], &stage_params[s][k], "stage_params")) return rc;
            if (int rc = check_grads(bd.stage[s], &stage_grads[s][k], "stage_grads")) return rc;
        }
        if (s + 1 < bd.stages) {
            if (int rc = check_down_params(bd.down[s], &down_params[s])) return rc;
            if (int rc = check_down_grads(bd.down[s], &down_grads[s])) return rc;
        }
        for (int r = 0; r < bd.stages; ++r)
            if (overlaps(&tops[s], &dtops[r])) return fail(RVN_ERR_ALIAS, "tops[%d] and dtops[%d] overlap", s, r);
    }
    const Geo g0{(int)n, (int)h, (int)w};
    const size_t need = body_ws_bytes(bd, g0, true);
    if (int rc = check_ws(ws, ws_bytes, need)) return rc;
    for (int s = 0; s < bd.stages; ++s)
        if (overlaps_range(&tops[s], ws, need) || overlaps_range(&dtops[s], ws, need))
            return fail(RVN_ERR_ALIAS, "tops[%d] or dtops[%d] overlaps the workspace", s, s);
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    const bool acc = accumulate_wgrads != 0;
    for (int s = bd.stages - 1; s >= 0; --s) {
        const Geo g{g0.n, g0.h >> s, g0.w >> s};
        if (s + 1 < bd.stages) {
            // dtops[s+1] now holds the derivative with respect to this block's output
            const DownPlan dp = make_down_plan(bd.down[s], g, true);
            down_backward(cx, bd.down[s], dp, bind(dp, ws, true), view_of(&tops[s]), view_of(&dtops[s + 1]), down_params[s],
                          view_of(&dtops[s]), down_grads[s], acc);
        }
        const Plan pl = make_plan(bd.stage[s], g, true);
        const View t1 = half_view(&tops[s], 0), t2 = half_view(&tops[s], 1);
        const View d1 = half_view(&dtops[s], 0), d2 = half_view(&dtops[s], 1);
        stack_backward(cx, bd.stage[s], bd.depth[s], pl, bind(pl, ws), g, t1, t2, d1, d2, stage_params[s], t1, t2, d1, d2,
                       stage_grads[s], acc);
    }
    return finish(cx);
}

// ---- fixed-point residual stream ---------------------------------------------

namespace {

int check_frac_bits(int32_t frac_bits) {
    if (frac_bits < 1 || frac_bits > 30) return fail(RVN_ERR_SHAPE, "frac_bits = %d out of range [1, 30]", frac_bits);
    return RVN_OK;
}

}  // namespace

int revnet_fixed_workspace_bytes(const rvn_block_desc *desc, int64_t n, int64_t h, int64_t w, size_t *fwd_bytes,
                                 size_t *bwd_bytes) {
    if (int rc = check_desc(desc)) return rc;
    if (int rc = check_geo(n, h, w)) return rc;
    const Geo g{(int)n, (int)h, (int)w};
    if (fwd_bytes) *fwd_bytes = make_plan(*desc, g, false, true).total;
    if (bwd_bytes) *bwd_bytes = make_plan(*desc, g, true, true).total;
    return RVN_OK;
}

int revnet_fixed_from_float(const rvn_tensor *src, int32_t frac_bits, const rvn_tensor *dst, void *hip_stream) {
    if (int rc = check_frac_bits(frac_bits)) return rc;
    if (!src) return fail(RVN_ERR_NULL, "tensor src is NULL");
    if (int rc = check_any_tensor("src", src, src->c, src->n, src->h, src->w)) return rc;
    if (int rc = check_any_tensor("dst", dst, src->c, src->n, src->h, src->w)) return rc;
    if (!same_tensor(src, dst) && overlaps(src, dst)) return fail(RVN_ERR_ALIAS, "src and dst overlap");
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    fix_from_float(cx, view_of(src), (int)src->c, Geo{(int)src->n, (int)src->h, (int)src->w}, frac_bits, view_of(dst));
    return finish(cx);
}

int revnet_fixed_to_float(const rvn_tensor *src, int32_t frac_bits, const rvn_tensor *dst, void *hip_stream) {
    if (int rc = check_frac_bits(frac_bits)) return rc;
    if (!src) return fail(RVN_ERR_NULL, "tensor src is NULL");
    if (int rc = check_any_tensor("src", src, src->c, src->n, src->h, src->w)) return rc;
    if (int rc = check_any_tensor("dst", dst, src->c, src->n, src->h, src->w)) return rc;
    if (dst->sc != dst->h * dst->w || dst->sn != dst->c * dst->sc)
        return fail(RVN_ERR_STRIDE, "tensor dst must be dense (sc = h*w, sn = c*h*w)");
    if (overlaps(src, dst)) return fail(RVN_ERR_ALIAS, "src and dst overlap");
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    fix_to_float(cx, view_of(src), (int)src->c, Geo{(int)src->n, (int)src->h, (int)src->w}, frac_bits,
                 static_cast<float *>(dst->ptr));
    return finish(cx);
}

int revnet_stack_fwd_fixed(const rvn_block_desc *desc, int32_t depth, int32_t frac_bits, const rvn_tensor *x1,
                           const rvn_tensor *x2, const rvn_block_params *params, const rvn_tensor *y1,
                           const rvn_tensor *y2, void *ws, size_t ws_bytes, void *hip_stream) {
    Plan pl;
    Geo g;
    if (depth <= 0) return fail(RVN_ERR_SHAPE, "depth = %d must be positive", depth);
    if (int rc = check_frac_bits(frac_bits)) return rc;
    if (int rc = check_fwd_args(desc, x1, x2, y1, y2, ws, ws_bytes, &pl, &g, true)) return rc;
    if (!params) return fail(RVN_ERR_NULL, "params is NULL");
    for (int k = 0; k < depth; ++k)
        if (int rc = check_params(*desc, &params[k], "params")) return rc;
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    stack_forward(cx, *desc, depth, pl, bind(pl, ws), g, view_of(x1), view_of(x2), params, view_of(y1), view_of(y2),
                  frac_bits);
    return finish(cx);
}

int revnet_stack_bwd_fixed(const rvn_block_desc *desc, int32_t depth, int32_t frac_bits, const rvn_tensor *y1,
                           const rvn_tensor *y2, const rvn_tensor *dy1, const rvn_tensor *dy2,
                           const rvn_block_params *params, const rvn_tensor *x1, const rvn_tensor *x2,
                           const rvn_tensor *dx1, const rvn_tensor *dx2, const rvn_block_grads *grads,
                           int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream) {
    Plan pl;
    Geo g;
    if (depth <= 0) return fail(RVN_ERR_SHAPE, "depth = %d must be positive", depth);
    if (int rc = check_frac_bits(frac_bits)) return rc;
    if (int rc = check_bwd_args(desc, y1, y2, dy1, dy2, x1, x2, dx1, dx2, ws, ws_bytes, &pl, &g, true)) return rc;
    if (!params) return fail(RVN_ERR_NULL, "params is NULL");
    if (!grads) return fail(RVN_ERR_NULL, "grads is NULL");
    for (int k = 0; k < depth; ++k) {
        if (int rc = check_params(*desc, &params[k], "params")) return rc;
        if (int rc = check_grads(*desc, &grads[k], "grads")) return rc;
    }
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    stack_backward(cx, *desc, depth, pl, bind(pl, ws), g, view_of(y1), view_of(y2), view_of(dy1), view_of(dy2), params,
                   view_of(x1), view_of(x2), view_of(dx1), view_of(dx2), grads, accumulate_wgrads != 0, frac_bits);
    return finish(cx);
}

// ---- stem ----------------------------------------------------------------------

namespace {

int check_stem(const rvn_stem_desc *d, int64_t n, int64_t h, int64_t w, StemShape *g) {
    if (!d) return fail(RVN_ERR_NULL, "descriptor is NULL");
    if (d->c_in <= 0 || d->c_out <= 0 || d->c_out > 65536) return fail(RVN_ERR_SHAPE, "c_in = %d, c_out = %d out of range", d->c_in, d->c_out);
    if (d->ks < 1 || d->ks > 7 || d->ks % 2 == 0 || (int64_t)d->c_in * d->ks * d->ks > 256)
        return fail(RVN_ERR_SHAPE, "ks = %d must be 1, 3, 5 or 7 with c_in * ks * ks <= 256 (c_in = %d)", d->ks, d->c_in);
    if (d->stride != 1 && d->stride != 2) return fail(RVN_ERR_SHAPE, "stride = %d must be 1 or 2", d->stride);
    if (int rc = check_geo(n, h, w)) return rc;
    *g = StemShape{(int)n, d->c_in, (int)h, (int)w, d->c_out, d->ks, d->stride, (int)((h - 1) / d->stride + 1),
                   (int)((w - 1) / d->stride + 1)};
    return RVN_OK;
}

struct StemPlan {
    // pooled derivative spread back to the convolution's output; the pooling windows' winners;
    // filter-gradient partial sums
    size_t dh, arg, part, total;
};

StemPlan make_stem_plan(const rvn_stem_desc &d, const StemShape &g) {
    StemPlan p{};
    size_t off = 0;
    p.dh = off;
    if (d.pool) off = align_up(off + (size_t)g.N * g.CO * g.HO * g.WO * 4);
    p.arg = off;
    if (d.pool) off = align_up(off + maxpool3s2_scratch_bytes(g.CO, Geo{g.N, g.HO, g.WO}));
    p.part = off;
    off = align_up(off + stem_wgrad_scratch_floats(g) * 4);
    p.total = off;
    return p;
}

}  // namespace

int revnet_stem_workspace_bytes(const rvn_stem_desc *desc, int64_t n, int64_t h, int64_t w, size_t *bwd_bytes) {
    StemShape g;
    if (int rc = check_stem(desc, n, h, w, &g)) return rc;
    if (bwd_bytes) *bwd_bytes = make_stem_plan(*desc, g).total;
    return RVN_OK;
}

int revnet_stem_fwd(const rvn_stem_desc *desc, const rvn_tensor *img, const float *w, const rvn_tensor *conv_out,
                    const rvn_tensor *y, void *hip_stream) {
    if (!img) return fail(RVN_ERR_NULL, "tensor img is NULL");
    StemShape g;
    if (int rc = check_stem(desc, img->n, img->h, img->w, &g)) return rc;
    if (int rc = check_any_tensor("img", img, g.CI, g.N, g.H, g.W)) return rc;
    if (!w) return fail(RVN_ERR_NULL, "w is NULL");
    const Geo mid{g.N, g.HO, g.WO};
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    if (!desc->pool) {
        if (conv_out) return fail(RVN_ERR_SHAPE, "conv_out must be NULL when pool == 0");
        if (int rc = check_any_tensor("y", y, g.CO, g.N, g.HO, g.WO)) return rc;
        if (overlaps(img, y)) return fail(RVN_ERR_ALIAS, "img and y overlap");
        stem_conv(cx, view_of(img), w, g, view_of(y));
        return finish(cx);
    }
    if (int rc = check_any_tensor("conv_out", conv_out, g.CO, g.N, g.HO, g.WO)) return rc;
    if (int rc = check_any_tensor("y", y, g.CO, g.N, (g.HO - 1) / 2 + 1, (g.WO - 1) / 2 + 1)) return rc;
    if (overlaps(img, y) || overlaps(img, conv_out) || overlaps(conv_out, y))
        return fail(RVN_ERR_ALIAS, "img, conv_out and y must not overlap");
    stem_conv(cx, view_of(img), w, g, view_of(conv_out));
    maxpool3s2_fwd(cx, view_of(conv_out), g.CO, mid, view_of(y));
    return finish(cx);
}

int revnet_stem_bwd(const rvn_stem_desc *desc, const rvn_tensor *img, const rvn_tensor *conv_out, const rvn_tensor *dy,
                    float *d_w, int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream) {
    if (!img) return fail(RVN_ERR_NULL, "tensor img is NULL");
    StemShape g;
    if (int rc = check_stem(desc, img->n, img->h, img->w, &g)) return rc;
    if (int rc = check_any_tensor("img", img, g.CI, g.N, g.H, g.W)) return rc;
    if (!d_w) return fail(RVN_ERR_NULL, "d_w is NULL");
    const StemPlan pl = make_stem_plan(*desc, g);
    if (int rc = check_ws(ws, ws_bytes, pl.total)) return rc;
    char *base = static_cast<char *>(ws);
    float *part = reinterpret_cast<float *>(base + pl.part);
    const Geo mid{g.N, g.HO, g.WO};
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    if (!desc->pool) {
        if (conv_out) return fail(RVN_ERR_SHAPE, "conv_out must be NULL when pool == 0");
        if (int rc = check_any_tensor("dy", dy, g.CO, g.N, g.HO, g.WO)) return rc;
        if (overlaps_range(img, ws, pl.total) || overlaps_range(dy, ws, pl.total))
            return fail(RVN_ERR_ALIAS, "a tensor overlaps the workspace");
        stem_wgrad(cx, view_of(img), view_of(dy), g, part, d_w, accumulate_wgrads != 0);
        return finish(cx);
    }
    if (int rc = check_any_tensor("conv_out", conv_out, g.CO, g.N, g.HO, g.WO)) return rc;
    if (int rc = check_any_tensor("dy", dy, g.CO, g.N, (g.HO - 1) / 2 + 1, (g.WO - 1) / 2 + 1)) return rc;
    if (overlaps_range(img, ws, pl.total) || overlaps_range(dy, ws, pl.total) || overlaps_range(conv_out, ws, pl.total))
        return fail(RVN_ERR_ALIAS, "a tensor overlaps the workspace");
    float *dh = reinterpret_cast<float *>(base + pl.dh);
    maxpool3s2_bwd(cx, view_of(conv_out), view_of(dy), g.CO, mid, reinterpret_cast<unsigned char *>(base + pl.arg), dh);
    stem_wgrad(cx, view_of(img), dense_view(dh, g.CO, mid), g, part, d_w, accumulate_wgrads != 0);
    return finish(cx);
}

}  // extern "C"
