// Host side of the non-reversible subsampling block and of the multi-stage
// body (reversible stages joined by such blocks): validation, workspace
// planning and the drivers that sequence the HIP kernels.
#include <algorithm>
#include <cstdio>

#include "api_common.h"

using namespace rvn;
using namespace rvn::api;

namespace {

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
    const int kind = enum_bits(d->kind), conv_dtype = enum_bits(d->conv_dtype);
    if (kind != RVN_BASIC && kind != RVN_BOTTLENECK) return fail(RVN_ERR_DTYPE, "unknown block kind %d", kind);
    if (conv_dtype != RVN_F32 && conv_dtype != RVN_BF16) return fail(RVN_ERR_DTYPE, "unknown conv_dtype %d", conv_dtype);
    if (d->c_in <= 0 || d->c_in > 131072 || d->c_out <= 0 || d->c_out > 131072)
        return fail(RVN_ERR_SHAPE, "c_in = %d, c_out = %d out of range [1, 131072]", d->c_in, d->c_out);
    if (kind == RVN_BOTTLENECK && (d->width <= 0 || d->width > 65536))
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
        if (ks == 3) cv_s = std::max(cv_s, conv3x3_bf16_scratch_floats(cin, cout, g, 2));  // (the strided layer's forward)
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

// With recompute_only the internals (statistics, h_l, subsampled x) are left
// in `b` for down_backward and y is not formed.
void down_forward(Ctx &cx, const rvn_down_desc &d, const DownPlan &pl, const DownBufs &b, View x,
                  const rvn_down_params &p, View y, bool recompute_only) {
    clear_counters(cx, b.counters, pl.n_counters);
    cx.emit_buf = nullptr;  // the statistics of this block's tensors are always read from the tensors
    cx.emit_floats = 0;
    // bf16 filters: one conversion launch per geometry (the order a 1x1 filter is stored in depends on
    // the geometry its layer runs at): the layers before and including the strided one, then the rest
    // and the shortcut.
    for (int pass = 0; pass < 2; ++pass) {
        FilterPrep fp[3];
        int nf = 0;
        const Geo &gp = pass == 0 ? pl.full : pl.low;
        for (int l = 0; l < pl.L; ++l) {
            const bool at_full = pl.gin[l].h == pl.full.h;
            if (at_full == (pass == 0))
                fp[nf++] = FilterPrep{p.R.conv_w[l], pl.layers[l].cin, pl.layers[l].cout, pl.layers[l].ks, b.wq_f[l], b.wq_b[l]};
        }
        if (pass == 1) fp[nf++] = FilterPrep{p.shortcut_w, d.c_in, d.c_out, 1, b.wq_f[kShortcut], b.wq_b[kShortcut]};
        if (nf == 0 || !pl.bf16) continue;
        double bytes = 0.0;
        const PrepArgs pa = plan_filter_prep(fp, nf, gp, &bytes);
        prep_filters_bf16(cx, pa, bytes);
    }
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
        } else if (ly.strided && ly.ks == 3 && d.conv_dtype == RVN_BF16 &&
                   conv3x3_bf16_stride2(cx, cur, scale_shift, b.wq_f[l], ly.cin, ly.cout, g, dense_view(b.h[l], ly.cout, pl.low),
                                        b.conv_scratch)) {
            cur = dense_view(b.h[l], ly.cout, pl.low);  // only the outputs that exist were computed
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
            const View xs = dense_view(b.xs, d.c_in, pl.low);
            WgradReduce sred;
            if (d.conv_dtype == RVN_BF16 &&
                conv_dgrad_wgrad_bf16(cx, xs, scale_shift, dy, nullptr, b.wq_b[kShortcut], d.c_in, d.c_out, 1, pl.low, b.wgrad_scratch,
                                      gr.d_shortcut_w, accumulate, b.t, b.conv_scratch, &sred)) {
                wgrad_reduce(cx, sred);
            } else {
                conv_wgrad(cx, xs, scale_shift, d.conv_dtype, dy, d.c_in, d.c_out, 1, pl.low, b.wgrad_scratch,
                           gr.d_shortcut_w, accumulate);
                conv_dgrad(cx, dy, d.conv_dtype, p.shortcut_w, b.wq_b[kShortcut], d.c_in, d.c_out, 1, pl.low, b.t,
                           b.conv_scratch);
            }
        }
        WgradReduce red;
        if (d.conv_dtype != RVN_BF16 ||
            !conv_dgrad_wgrad_bf16(cx, xl, scale_shift, dcur, nullptr, b.wq_b[l], ly.cin, ly.cout, ly.ks, g, b.wgrad_scratch,
                                   gr.R.d_conv_w[l], accumulate, da, b.conv_scratch, &red)) {
            conv_wgrad(cx, xl, scale_shift, d.conv_dtype, dcur, ly.cin, ly.cout, ly.ks, g, b.wgrad_scratch, gr.R.d_conv_w[l],
                       accumulate, &red);
            conv_dgrad(cx, dcur, d.conv_dtype, p.R.conv_w[l], b.wq_b[l], ly.cin, ly.cout, ly.ks, g, da, b.conv_scratch);
        }
        if (l == 0) upsample2_add(cx, b.t, d.c_in, pl.full, da);
        const View out = l == 0 ? dx : dense_view(da, ly.cin, g);
        bn_relu_bwd(cx, xl, da, ly.cin, g, b.stats[l], b.bn_scratch, b.counters, gr.R.d_bn_gamma[l], gr.R.d_bn_beta[l],
                    accumulate, nullptr, out, &red);
        dcur = out;
        cur ^= 1;
    }
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

// Workspace of a body call: the largest need of any stage or subsampling block.
// With a fixed-point stream two fp32 tensors follow it: the input of the
// subsampling block at hand (the stored top, decoded) and its output (before
// it is encoded into the next stage's tensor).
struct BodyWs {
    size_t plan, xin, yout, total;
};

BodyWs body_ws(const rvn_body_desc &bd, const Geo &g0, bool backward, bool fixed) {
    BodyWs w{};
    size_t in_max = 0, out_max = 0;
    for (int s = 0; s < bd.stages; ++s) {
        const Geo g{g0.n, g0.h >> s, g0.w >> s};
        w.plan = std::max(w.plan, make_plan(bd.stage[s], g, backward, fixed).total);
        if (s + 1 < bd.stages) {
            w.plan = std::max(w.plan, make_down_plan(bd.down[s], g, backward).total);
            in_max = std::max(in_max, (size_t)g.pixels() * bd.down[s].c_in * 4);
            out_max = std::max(out_max, (size_t)(g.pixels() / 4) * bd.down[s].c_out * 4);
        }
    }
    w.plan = align_up(w.plan);
    w.xin = w.plan;
    w.yout = w.xin + (fixed ? align_up(in_max) : 0);
    w.total = w.yout + (fixed ? align_up(out_max) : 0);
    return w;
}

size_t body_ws_bytes(const rvn_body_desc &bd, const Geo &g0, bool backward, bool fixed = false) {
    return body_ws(bd, g0, backward, fixed).total;
}

View half_view(const rvn_tensor *t, int which) {
    return View{static_cast<float *>(t->ptr) + (int64_t)which * (t->c / 2) * t->sc, t->sn, t->sc};
}

}  // namespace

extern "C" {

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

namespace {

// frac_bits > 0: the tops hold fixed-point codes (x is fp32 and is encoded into
// tops[0]; every subsampling block reads the decoded top and its fp32 output is
// encoded into the next stage's tensor).
int body_fwd_impl(const rvn_body_desc *desc, const rvn_tensor *x, const rvn_block_params *const *stage_params,
                  const rvn_down_params *down_params, const rvn_tensor *tops, void *ws, size_t ws_bytes,
                  void *hip_stream, int frac_bits) {
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
    const BodyWs bw = body_ws(bd, g0, false, frac_bits != 0);
    const size_t need = bw.total;
    if (int rc = check_ws(ws, ws_bytes, need)) return rc;
    if (overlaps_range(x, ws, need)) return fail(RVN_ERR_ALIAS, "x overlaps the workspace");
    for (int s = 0; s < bd.stages; ++s)
        if (overlaps_range(&tops[s], ws, need)) return fail(RVN_ERR_ALIAS, "tops[%d] overlaps the workspace", s);
    Ctx cx;
    cx.stream = static_cast<hipStream_t>(hip_stream);
    for (int s = 0; s < bd.stages; ++s) {
        const Geo g{g0.n, g0.h >> s, g0.w >> s};
        const Plan pl = make_plan(bd.stage[s], g, false, frac_bits != 0);
        const rvn_tensor *in = s == 0 ? x : &tops[s];  // later stages run in place on the subsampling block's output
        if (frac_bits && s == 0) {
            fix_from_float(cx, view_of(x), (int)x->c, g, frac_bits, view_of(&tops[0]));
            in = &tops[0];
        }
        stack_forward(cx, bd.stage[s], bd.depth[s], pl, bind(pl, ws), g, half_view(in, 0), half_view(in, 1),
                      stage_params[s], half_view(&tops[s], 0), half_view(&tops[s], 1), frac_bits);
        if (s + 1 < bd.stages) {
            const DownPlan dp = make_down_plan(bd.down[s], g, false);
            if (frac_bits) {
                char *base = static_cast<char *>(ws);
                float *xin = reinterpret_cast<float *>(base + bw.xin), *yout = reinterpret_cast<float *>(base + bw.yout);
                const Geo low{g.n, g.h / 2, g.w / 2};
                fix_to_float(cx, view_of(&tops[s]), bd.down[s].c_in, g, frac_bits, xin);
                const View yv = dense_view(yout, bd.down[s].c_out, low);
                down_forward(cx, bd.down[s], dp, bind(dp, ws, false), dense_view(xin, bd.down[s].c_in, g), down_params[s], yv,
                             false);
                fix_from_float(cx, yv, bd.down[s].c_out, low, frac_bits, view_of(&tops[s + 1]));
            } else {
                down_forward(cx, bd.down[s], dp, bind(dp, ws, false), view_of(&tops[s]), down_params[s],
                             view_of(&tops[s + 1]), false);
            }
        }
    }
    return finish(cx);
}

}  // namespace

int revnet_body_fwd(const rvn_body_desc *desc, const rvn_tensor *x, const rvn_block_params *const *stage_params,
                    const rvn_down_params *down_params, const rvn_tensor *tops, void *ws, size_t ws_bytes,
                    void *hip_stream) {
    return body_fwd_impl(desc, x, stage_params, down_params, tops, ws, ws_bytes, hip_stream, 0);
}

int revnet_body_fwd_fixed(const rvn_body_desc *desc, int32_t frac_bits, const rvn_tensor *x,
                          const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                          const rvn_tensor *tops, void *ws, size_t ws_bytes, void *hip_stream) {
    if (frac_bits < 1 || frac_bits > 30) return fail(RVN_ERR_SHAPE, "frac_bits = %d out of range [1, 30]", frac_bits);
    return body_fwd_impl(desc, x, stage_params, down_params, tops, ws, ws_bytes, hip_stream, frac_bits);
}



namespace {

int body_bwd_impl(const rvn_body_desc *desc, const rvn_tensor *tops, const rvn_tensor *dtops,
                  const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                  const rvn_block_grads *const *stage_grads, const rvn_down_grads *down_grads,
                  int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream, int frac_bits) {
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
    const BodyWs bw = body_ws(bd, g0, true, frac_bits != 0);
    const size_t need = bw.total;
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
            View xin = view_of(&tops[s]);
            if (frac_bits) {  // the stored input, decoded
                float *xf = reinterpret_cast<float *>(static_cast<char *>(ws) + bw.xin);
                fix_to_float(cx, xin, bd.down[s].c_in, g, frac_bits, xf);
                xin = dense_view(xf, bd.down[s].c_in, g);
            }
            down_backward(cx, bd.down[s], dp, bind(dp, ws, true), xin, view_of(&dtops[s + 1]), down_params[s],
                          view_of(&dtops[s]), down_grads[s], acc);
        }
        const Plan pl = make_plan(bd.stage[s], g, true, frac_bits != 0);
        const View t1 = half_view(&tops[s], 0), t2 = half_view(&tops[s], 1);
        const View d1 = half_view(&dtops[s], 0), d2 = half_view(&dtops[s], 1);
        stack_backward(cx, bd.stage[s], bd.depth[s], pl, bind(pl, ws), g, t1, t2, d1, d2, stage_params[s], t1, t2, d1, d2,
                       stage_grads[s], acc, frac_bits);
    }
    return finish(cx);
}

}  // namespace

int revnet_body_bwd(const rvn_body_desc *desc, const rvn_tensor *tops, const rvn_tensor *dtops,
                    const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                    const rvn_block_grads *const *stage_grads, const rvn_down_grads *down_grads,
                    int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream) {
    return body_bwd_impl(desc, tops, dtops, stage_params, down_params, stage_grads, down_grads, accumulate_wgrads, ws,
                         ws_bytes, hip_stream, 0);
}

int revnet_body_bwd_fixed(const rvn_body_desc *desc, int32_t frac_bits, const rvn_tensor *tops, const rvn_tensor *dtops,
                          const rvn_block_params *const *stage_params, const rvn_down_params *down_params,
                          const rvn_block_grads *const *stage_grads, const rvn_down_grads *down_grads,
                          int accumulate_wgrads, void *ws, size_t ws_bytes, void *hip_stream) {
    if (frac_bits < 1 || frac_bits > 30) return fail(RVN_ERR_SHAPE, "frac_bits = %d out of range [1, 30]", frac_bits);
    return body_bwd_impl(desc, tops, dtops, stage_params, down_params, stage_grads, down_grads, accumulate_wgrads, ws,
                         ws_bytes, hip_stream, frac_bits);
}

int revnet_body_fixed_workspace_bytes(const rvn_body_desc *desc, int64_t n, int64_t h, int64_t w, size_t *fwd_bytes,
                                      size_t *bwd_bytes) {
    if (int rc = check_body_desc(desc, n, h, w)) return rc;
    const Geo g{(int)n, (int)h, (int)w};
    if (fwd_bytes) *fwd_bytes = body_ws_bytes(*desc, g, false, true);
    if (bwd_bytes) *bwd_bytes = body_ws_bytes(*desc, g, true, true);
    return RVN_OK;
}



}  // extern "C"
