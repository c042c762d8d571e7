// Host side of the stem (image convolution, max-pooling): validation, workspace
// planning and the launches.
#include "api_common.h"

using namespace rvn;
using namespace rvn::api;

extern "C" {

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
