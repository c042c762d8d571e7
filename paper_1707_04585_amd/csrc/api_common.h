// Host-side helpers shared by the entry points of the library (block / stack,
// subsampling block / body, stem): error reporting, argument checks, the
// workspace plan of a reversible stack and its drivers.  Not part of the
// public ABI (that is include/revnet.h).
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "kernels.h"

namespace rvn {
namespace api {

// Records the message for revnet_last_error (thread local) and returns `code`.
int fail(int code, const char *fmt, ...);
const char *last_error();
// cx.err as a status of the ABI.
int finish(Ctx &cx);

// The integer a caller put into an enum field.  Read as bytes: a value outside
// the enumerators' range must be reported, and loading it through the enum
// type would be undefined behaviour in C++.
template <typename E>
inline int enum_bits(const E &field) {
    static_assert(sizeof(E) == sizeof(int), "enum fields of the ABI are int-sized");
    int v;
    __builtin_memcpy(&v, &field, sizeof v);
    return v;
}

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// ---- argument checks (all before the first launch) --------------------------
int check_desc(const rvn_block_desc *d);
int check_geo(int64_t n, int64_t h, int64_t w);
int check_ws(const void *ws, size_t have, size_t need);
int check_params(const rvn_block_desc &d, const rvn_block_params *p, const char *what);
int check_grads(const rvn_block_desc &d, const rvn_block_grads *p, const char *what);
// Shape [n, c, h, w], the supported strides (sw = 1, sh = w, sc >= h*w, sn >= (c-1)*sc + h*w), alignment.
int check_any_tensor(const char *name, const rvn_tensor *t, int64_t c, int64_t n, int64_t h, int64_t w);
bool same_tensor(const rvn_tensor *a, const rvn_tensor *b);
bool overlaps(const rvn_tensor *a, const rvn_tensor *b);
bool overlaps_range(const rvn_tensor *a, const void *p, size_t bytes);
View view_of(const rvn_tensor *t);

// ---- reversible stacks ----------------------------------------------------------
struct Layer {
    int cin, cout, ks;
};
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
    // per-tile statistics that a 1x1 bf16 convolution leaves for the BN layer reading its output
    size_t emit, emit_floats;
    // two spare layer-0 statistics arrays: a function's input statistics that a launch of the
    // backward pass computed ahead (merge of the producing convolution's partial results)
    size_t stats_in[2];
    size_t total;
};
struct Bufs {
    float *stats[3];
    float *h[2];
    float *g[2];
    float *bn_scratch;
    float *wgrad_scratch, *conv_scratch;
    int *counters;
    uint16_t *wq_f[3], *wq_b[3];  // null where the layer does not use converted filters
    float *xf, *fout;
    float *emit;  // null when the plan has none
    float *stats_in[2];
};
Plan make_plan(const rvn_block_desc &d, const Geo &g, bool backward, bool fixed = false);
Bufs bind(const Plan &p, void *ws);
// All argument checks of a forward call (descriptor, the four tensors, aliasing, workspace size,
// alignment and overlap); on success *plan and *geo describe the call.
int check_fwd_args(const rvn_block_desc *desc, const rvn_tensor *x1, const rvn_tensor *x2, const rvn_tensor *y1,
                   const rvn_tensor *y2, void *ws, size_t ws_bytes, Plan *plan, Geo *geo, bool fixed);

// Section 3.2: blocks params[0 .. depth-1] in order, only the top pair kept; and
// Algorithm 1 applied from the top block down.  frac_bits > 0: the stream
// tensors hold fixed-point codes.
void stack_forward(Ctx &cx, const rvn_block_desc &d, int depth, const Plan &pl, const Bufs &b, Geo g, View x1, View x2,
                   const rvn_block_params *params, View y1, View y2, int frac_bits = 0);
void stack_backward(Ctx &cx, const rvn_block_desc &d, int depth, const Plan &pl, const Bufs &b, Geo g, View y1, View y2,
                    View dy1, View dy2, const rvn_block_params *params, View x1, View x2, View dx1, View dx2,
                    const rvn_block_grads *grads, bool accumulate, int frac_bits = 0);

}  // namespace api
}  // namespace rvn
