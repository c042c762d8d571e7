// Host side of the library: argument validation, workspace planning and the
// block / stack drivers that sequence the HIP kernels.  Everything here runs
// on the host and only enqueues work on the caller's stream.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "api_common.h"


namespace rvn {
namespace api {


thread_local char g_err[512] = "";

const char *last_error() { return g_err; }

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}


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
    const int kind = enum_bits(d->kind), conv_dtype = enum_bits(d->conv_dtype);
    if (kind != RVN_BASIC && kind != RVN_BOTTLENECK) return fail(RVN_ERR_DTYPE, "unknown block kind %d", kind);
    if (conv_dtype != RVN_F32 && conv_dtype != RVN_BF16) return fail(RVN_ERR_DTYPE, "unknown conv_dtype %d", conv_dtype);
    if (d->c_half <= 0 || d->c_half > 65536)
        return fail(RVN_ERR_SHAPE, "c_half = %d out of range [1, 65536]", d->c_half);
    if (kind == RVN_BOTTLENECK && (d->width <= 0 || d->width > 65536))
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



// Filters this large are converted once per function evaluation instead of in
// every workgroup of the convolution.
bool wants_prep(const rvn_block_desc &d, const Layer &ly, const Geo &g) {
    if (d.conv_dtype != RVN_BF16) return false;
    if (ly.ks == 1 && (conv1x1_direct_ok(ly.cin, g) || conv1x1_direct_ok(ly.cout, g))) return true;
    if (ly.ks == 3 && (conv3x3_bf16_ok(ly.cin, ly.cout, g) || conv3x3_bf16_ok(ly.cout, ly.cin, g))) return true;
    return (int64_t)ly.cin * ly.cout * ly.ks * ly.ks >= 16384;
}

Plan make_plan(const rvn_block_desc &d, const Geo &g, bool backward, bool fixed) {
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
    {
        // (mean, M2) per channel and pixel tile of a convolution's output: 128-pixel tiles of the bf16
        // 1x1 kernel, 64-pixel wavefront shares of the 3x3 kernels
        const size_t tiles128 = ((size_t)g.n * (((size_t)g.h * g.w + 3) / 4) + 31) / 32, tiles64 = P / 64 + kAlign;
        for (int l = 0; l < p.L; ++l) {
            const Layer &ly = p.layers[l];
            if (d.conv_dtype == RVN_BF16 && ly.ks == 1) p.emit_floats = std::max(p.emit_floats, (size_t)ly.cout * tiles128 * 2);
            if (ly.ks == 3 && (d.conv_dtype == RVN_BF16 || ly.cout <= 32))
                p.emit_floats = std::max(p.emit_floats, (size_t)ly.cout * tiles64 * 2);
        }
        p.emit = off;
        off = align_up(off + p.emit_floats * 4);
    }
    for (int i = 0; i < 2; ++i) {
        p.stats_in[i] = off;
        off = align_up(off + kStatsArrays * (size_t)p.layers[0].cin * 4);
    }
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
    o.emit = p.emit_floats ? reinterpret_cast<float *>(b + p.emit) : nullptr;
    for (int i = 0; i < 2; ++i) o.stats_in[i] = reinterpret_cast<float *>(b + p.stats_in[i]);
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
// Returns where the statistics of layer 0 are: b.stats[0], or the spare array that a carried merge
// filled ahead (see arm_merge); func_backward of the same function must be given that pointer.
const float *func_forward(Ctx &cx, const rvn_block_desc &d, const Plan &pl, const Bufs &b, Geo g, View x,
                          const rvn_func_params &p, Epilogue ep, const View *r, View out, int frac_bits) {
    // the input's statistics may be there already
    const EmittedStats pm = cx.premerged;
    const float *const pm_stats = cx.premerged_stats;
    cx.premerged = EmittedStats{};
    cx.premerged_stats = nullptr;
    const bool ahead = !frac_bits && pm.p && pm_stats && pm.p == x.p && pm.sn == x.sn && pm.sc == x.sc &&
                       pm.c == pl.layers[0].cin && pm.n == g.n && pm.h == g.h && pm.w == g.w;
    const float *const stats0 = ahead ? pm_stats : b.stats[0];
    View cur = x;
    // Convolutions leave statistics of their output for the next BN layer.  With the fixed-point
    // stream only the inner tensors of a function can use them; that pays for the three-layer
    // function (-1 % at the bottleneck workload) and not for the two-layer one (+0.5 %).
    cx.emit_buf = frac_bits && pl.L < 3 ? nullptr : b.emit;
    cx.emit_floats = pl.emit_floats;
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
        if (l == 0 && ahead) {
            cx.emitted = EmittedStats{};  // (the filters were converted in the launch that merged the statistics)
        } else {
            bn_stats(cx, cur, ly.cin, g, d.bn_eps, p.bn_gamma[l], p.bn_beta[l], b.bn_scratch, b.counters, b.stats[l],
                     l == 0 && pa.jobs > 0 ? &pa : nullptr, l == 0 ? prep_bytes : 0.0);
        }
        const float *scale_shift = (l == 0 ? stats0 : b.stats[l]) + 2 * ly.cin;
        if (l < pl.L - 1) {
            View h = dense_view(b.h[l], ly.cout, g);
            conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, EP_STORE, nullptr, h, b.conv_scratch);
            cur = h;
        } else if (frac_bits) {
            // (no statistics from this epilogue: the next BN layer reads the stream's fp32 copy, not fout)
            float *const lent = cx.emit_buf;
            cx.emit_buf = nullptr;
            conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, EP_STORE, nullptr,
                     dense_view(b.fout, ly.cout, g), b.conv_scratch);
            cx.emit_buf = lent;
            fix_axpy(cx, *r, b.fout, ly.cout, g, frac_bits, ep == EP_SUB ? -1 : 1, out);
        } else {
            conv_fwd(cx, cur, scale_shift, d.conv_dtype, p.conv_w[l], b.wq_f[l], ly.cin, ly.cout, ly.ks, g, ep, r, out, b.conv_scratch);
        }
    }
    return stats0;
}

// If the convolution that has just run left partial statistics of `t` (the input of a function that
// runs only after the backward pass of another), let the last launch of that backward pass merge them
// into a spare statistics array with that function's layer-0 parameters; func_forward finds them
// there.  The conversion of that function's filters to bf16, which the replaced statistics launch
// would have carried, rides in the same launch.  Only with the floating-point stream.
void arm_merge(Ctx &cx, const rvn_block_desc &d, const Plan &pl, const Bufs &b, Geo g, View t,
               const rvn_func_params &consumer, int frac_bits) {
    const EmittedStats e = cx.emitted;
    const int c = pl.layers[0].cin;
    if (frac_bits || !cx.emit_buf || !e.p || e.count <= 0) return;
    if (e.p != t.p || e.sn != t.sn || e.sc != t.sc || e.c != c || e.n != g.n || e.h != g.h || e.w != g.w) return;
    float *const slot = b.stats_in[cx.premerge_slot];
    cx.premerge_slot ^= 1;
    StatsMerge m;
    m.partials = cx.emit_buf;
    m.tiles = e.tiles;
    m.count = (float)e.count;
    m.gamma = consumer.bn_gamma[0];
    m.beta = consumer.bn_beta[0];
    m.stats = slot;
    m.C = c;
    m.eps = d.bn_eps;
    m.blocks = c;
    cx.merge_carry = m;
    // the statistics launch this replaces would have carried the conversion of the consumer's filters
    FilterPrep prep[3];
    for (int l = 0; l < pl.L; ++l)
        prep[l] = FilterPrep{consumer.conv_w[l], pl.layers[l].cin, pl.layers[l].cout, pl.layers[l].ks, b.wq_f[l], b.wq_b[l]};
    double prep_bytes = 0.0;
    cx.prep_carry = plan_filter_prep(prep, pl.L, g, &prep_bytes);
    cx.premerged = e;
    cx.premerged_stats = slot;
    cx.emitted = EmittedStats{};
}

// Ordinary backprop through Func at the activations func_forward left in `b`
// (Section 2.1, the backprop rule): out = skip + (dFunc/dx)^T upstream, and
// the parameter gradients.
void func_backward(Ctx &cx, const rvn_block_desc &d, const Plan &pl, const Bufs &b, Geo g, View x,
                   const rvn_func_params &p, View upstream, const rvn_func_grads &gr, bool accumulate,
                   View skip, View out, const float *stats0) {
    View dh = upstream;
    const uint16_t *dh16 = nullptr;  // the upstream gradient of the layer at hand as bf16, when the layer above left it so
    int cur = 0;
    for (int l = pl.L - 1; l >= 0; --l) {
        const Layer &ly = pl.layers[l];
        const float *const st = l == 0 ? stats0 : b.stats[l];
        const View xl = l > 0 ? dense_view(b.h[l - 1], ly.cin, g) : x;
        // The ordered sum of the filter gradient's partial results rides in the
        // BN-backward apply launch below.
        WgradReduce red;
        float *da = b.g[cur];
        const bool paired =
            d.conv_dtype == RVN_F32
                ? conv_dgrad_wgrad_f32(cx, xl, st + 2 * ly.cin, dh, p.conv_w[l], ly.cin, ly.cout, ly.ks, g,
                                       b.wgrad_scratch, gr.d_conv_w[l], accumulate, da, &red)
                : conv_dgrad_wgrad_bf16(cx, xl, st + 2 * ly.cin, dh, dh16, b.wq_b[l], ly.cin, ly.cout, ly.ks, g,
                                        b.wgrad_scratch, gr.d_conv_w[l], accumulate, da, b.conv_scratch, &red);
        if (!paired) {
            if (dh16) {  // cannot happen: the layer above asked before it wrote bf16
                cx.fail(hipErrorInvalidValue);
                return;
            }
            conv_wgrad(cx, xl, st + 2 * ly.cin, d.conv_dtype, dh, ly.cin, ly.cout, ly.ks, g, b.wgrad_scratch,
                       gr.d_conv_w[l], accumulate, &red);
            conv_dgrad(cx, dh, d.conv_dtype, p.conv_w[l], b.wq_b[l], ly.cin, ly.cout, ly.ks, g, da, b.conv_scratch);
        }
        if (l > 0) {
            View dx = dense_view(da, ly.cin, g);
            // The gradient this BN backward produces is read only by the two gradient kernels of the layer
            // below, which round it to bf16 on load: where their shared launch takes it that way, it is
            // written rounded (same bits downstream, half the bytes three times over), into the other
            // ping-pong buffer, whose content (this layer's upstream gradient) is dead by now.
            const Layer &below = pl.layers[l - 1];
            const View x_below = l - 1 > 0 ? dense_view(b.h[l - 2], below.cin, g) : x;
            uint16_t *const as16 = reinterpret_cast<uint16_t *>(b.g[cur ^ 1]);
            const bool to16 = d.conv_dtype == RVN_BF16 && g.hw() % 4 == 0 &&
                              conv_dgrad_wgrad_takes_bf16_dh(x_below, as16, b.wq_b[l - 1], below.cin, below.cout, below.ks, g,
                                                             b.wgrad_scratch, da, b.conv_scratch);
            bn_relu_bwd(cx, xl, da, ly.cin, g, st, b.bn_scratch, b.counters, gr.d_bn_gamma[l], gr.d_bn_beta[l],
                        accumulate, nullptr, dx, &red, to16 ? as16 : nullptr);
            if (to16) {
                dh16 = as16;  // (da of this layer is dead after the launch above: the next layer reuses b.g[cur])
            } else {
                dh = dx;
                dh16 = nullptr;
                cur ^= 1;
            }
        } else {
            // the last launch of this function's backward pass: every use of its converted filters is
            // behind it, so what arm_merge prepared for the next function can ride here
            cx.carry_now = true;
            bn_relu_bwd(cx, x, da, ly.cin, g, st, b.bn_scratch, b.counters, gr.d_bn_gamma[l], gr.d_bn_beta[l],
                        accumulate, &skip, out, &red);
            cx.carry_now = false;
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
                    View dx2, const rvn_block_grads &gr, bool accumulate, int frac_bits,
                    const rvn_func_params *below_G) {
    const View shadow = dense_view(b.xf, d.c_half, g);  // fp32 copy of the function input at hand
    // z1 = y1;  x2 = y2 - G(z1)
    const float *const sg = func_forward(cx, d, pl, b, g, y1, p.G, EP_SUB, &y2, x2, frac_bits);
    // (x2 is read next by F, after G's backward pass: its statistics can be merged in between)
    arm_merge(cx, d, pl, b, g, x2, p.F, frac_bits);
    // dz1 = dy1 + (dG/dz1)^T dy2;  dwG          (dx1 = dz1)
    func_backward(cx, d, pl, b, g, frac_bits ? shadow : y1, p.G, dy2, gr.G, accumulate, dy1, dx1, sg);
    // x1 = z1 - F(x2)
    const float *const sf = func_forward(cx, d, pl, b, g, x2, p.F, EP_SUB, &y1, x1, frac_bits);
    // (x1 is the y1 of the block below: its G reads it after F's backward pass)
    if (below_G) arm_merge(cx, d, pl, b, g, x1, *below_G, frac_bits);
    // dx2 = dy2 + (dF/dx2)^T dz1;  dwF
    func_backward(cx, d, pl, b, g, frac_bits ? shadow : x2, p.F, dx1, gr.F, accumulate, dy2, dx2, sf);
}

int finish(Ctx &cx) {
    if (cx.err != hipSuccess) return fail(RVN_ERR_HIP, "HIP error: %s", hipGetErrorString(cx.err));
    return RVN_OK;
}

int check_fwd_args(const rvn_block_desc *desc, const rvn_tensor *x1, const rvn_tensor *x2,
                   const rvn_tensor *y1, const rvn_tensor *y2, void *ws, size_t ws_bytes, Plan *plan, Geo *geo,
                   bool fixed) {
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
                   bool fixed) {
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
                   View x1, View x2, const rvn_block_params *params, View y1, View y2, int frac_bits) {
    clear_counters(cx, b.counters, pl.n_counters);
    for (int k = 0; k < depth; ++k) {
        block_forward(cx, d, pl, b, g, k ? y1 : x1, k ? y2 : x2, params[k], y1, y2, frac_bits);
    }
}

void stack_backward(Ctx &cx, const rvn_block_desc &d, int depth, const Plan &pl, const Bufs &b, Geo g,
                    View y1, View y2, View dy1, View dy2, const rvn_block_params *params, View x1, View x2,
                    View dx1, View dx2, const rvn_block_grads *grads, bool accumulate, int frac_bits) {
    clear_counters(cx, b.counters, pl.n_counters);
    for (int k = depth - 1; k >= 0; --k) {
        const bool top = k == depth - 1;
        block_backward(cx, d, pl, b, g, top ? y1 : x1, top ? y2 : x2, top ? dy1 : dx1, top ? dy2 : dx2,
                       params[k], x1, x2, dx1, dx2, grads[k], accumulate, frac_bits, k > 0 ? &params[k - 1].G : nullptr);
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

}  // namespace api
}  // namespace rvn

using namespace rvn;
using namespace rvn::api;

extern "C" {

int revnet_version(void) { return 1000; }

const char *revnet_last_error(void) { return last_error(); }

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
    if (int rc = check_fwd_args(desc, x1, x2, y1, y2, ws, ws_bytes, &pl, &g, false)) return rc;
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
    if (int rc = check_bwd_args(desc, y1, y2, dy1, dy2, x1, x2, dx1, dx2, ws, ws_bytes, &pl, &g, false)) return rc;
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
    // (non-null: the drivers form addresses from these bases, and offsetting a null pointer is undefined)
    void *const placeholder_ws = reinterpret_cast<void *>(uintptr_t{1} << 40);
    const View v = dense_view(reinterpret_cast<float *>(uintptr_t{1} << 41), desc->c_half, g);
    if (fwd) {
        const Plan pl = make_plan(*desc, g, false);
        Ctx cx;
        cx.dry = true;
        stack_forward(cx, *desc, depth, pl, bind(pl, placeholder_ws), g, v, v, params.data(), v, v);
        *fwd = cx.cost;
    }
    if (bwd) {
        const Plan pl = make_plan(*desc, g, true);
        Ctx cx;
        cx.dry = true;
        stack_backward(cx, *desc, depth, pl, bind(pl, placeholder_ws), g, v, v, v, v, params.data(), v, v, v, v,
                       grads.data(), false);
        *bwd = cx.cost;
    }
    return RVN_OK;
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

}  // extern "C"
