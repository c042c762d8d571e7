// Internal interface between the host-side block/stack driver and the HIP
// kernels.  Not part of the public ABI (that is include/revnet.h).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "revnet.h"

namespace rvn {

// fp32 tensor whose rows and planes are contiguous: element (n, c, i), with
// i = row * W + col in [0, H*W), lives at p[n*sn + c*sc + i].
struct View {
    float *p;
    int64_t sn, sc;
};

struct Geo {
    int n, h, w;
    int hw() const { return h * w; }
    int64_t pixels() const { return (int64_t)n * h * w; }
};

inline View dense_view(float *p, int c, const Geo &g) {
    return View{p, (int64_t)c * g.hw(), (int64_t)g.hw()};
}

// What the last convolution of a residual function does with its sums
// (Section 3.1): plain store, r + acc (forward coupling) or r - acc
// (reconstruction).
enum Epilogue { EP_STORE = 0, EP_ADD = 1, EP_SUB = 2 };

// Kernel families, for launch accounting and the optional event profiler.
enum KernelId {
    K_BN_STATS = 0,
    K_CLEAR_COUNTERS,
    K_CONV_FWD,
    K_CONV_DGRAD,
    K_CONV_WGRAD,
    K_WGRAD_REDUCE,
    K_BN_BWD_REDUCE,
    K_BN_BWD_APPLY,
    K_PREP_FILTER,
    K_CONV_DGRAD_WGRAD,
    K_RESAMPLE,
    K_FIXED_POINT,
    K_STEM,
    K_SPLITK_REDUCE,  // second launch of a convolution whose input channels were split over workgroups
    K_COUNT
};
const char *kernel_name(int id);

// Optional per-launch timing (revnet_profile_begin / revnet_profile_end): a
// pair of HIP events that the launch itself stamps with the kernel's start and
// end on the stream it runs on.
void profile_new_mark(int id, double bytes, double flops, hipEvent_t *start, hipEvent_t *stop);
bool profile_enabled();

// Per-channel (mean, M2) of every pixel tile (128 or 64 pixels) of a tensor, written by the
// convolution that produced it; the next statistics pass of exactly that tensor
// merges them instead of reading the tensor again.
struct EmittedStats {
    const float *p = nullptr;  // the tensor: base, strides, channels, geometry
    int64_t sn = 0, sc = 0;
    int c = 0, n = 0, h = 0, w = 0;
    int tiles = 0;  // partial results per channel: partials[(channel * tiles + tile) * 2 + {0, 1}]
    int count = 0;  // pixels behind every partial result
};

// The filter w [cout][cin][ks][ks] in bf16 and in the order the bf16 kernel
// consumes it: qf [cout][ks*ks][cin padded to 8] for the forward convolution and
// (if qb != nullptr) qb [cin][ks*ks][cout padded to 8], transposed and flipped,
// for the data gradient.  filter_bf16_elems(rows, k_channels, ks) = elements of
// such a buffer.
//
// 1x1 filters whose reduction length (cin forward, cout for the data gradient)
// passes conv1x1_direct_ok are stored instead in the operand order of
// conv1x1_bf16: [rows / 32][k_channels / 16][64 lanes][8], zero padded.
size_t filter_bf16_elems(int rows, int k_channels, int ks);
struct FilterPrep {
    const float *w;  // [cout][cin][ks][ks]
    int cin, cout, ks;
    uint16_t *qf, *qb;  // destinations (either may be null)
};
// The conversion of the filters of up to three layers as one list of jobs
// (see prep_filter.h); plan_filter_prep builds it, prep_filters_bf16 runs it in
// a launch of its own, bn_stats can carry it instead.
struct PrepJob {
    const float *w;  // [CO][CI][KS2]
    uint16_t *q;
    int CO, CI, KS2, kind;
    int KP;      // channel pitch (kinds 0, 1) or 16-channel steps per row tile (kinds 2, 3)
    int block0;  // first workgroup of this job
    int64_t n;   // threads: elements to write (kinds 2, 3) or (row, padded column) pairs (kinds 0, 1)
};
struct PrepArgs {
    PrepJob job[6];
    int jobs, blocks;
};
// A merge of such partial results into the four per-channel statistics arrays
// (what bn_stats_merge_k does), as work that another launch can carry:
// `blocks` workgroups of 256 threads, one per channel; 0 = nothing.
struct StatsMerge {
    const float *partials = nullptr;
    int tiles = 0;
    float count = 0.f;
    const float *gamma = nullptr, *beta = nullptr;
    float *stats = nullptr;
    int C = 0;
    float eps = 0.f;
    int blocks = 0;
};

// One call's launch context.  With dry == true the wrappers only count.
struct Ctx {
    // A merge waiting for a launch to carry it (the apply launch of a BN-backward call made with carry_now), and the
    // record of a tensor whose statistics such a carried merge has put into `premerged_stats`.
    StatsMerge merge_carry;
    PrepArgs prep_carry = {};  // the filter conversion of the function that will read those statistics
    bool carry_now = false;    // set around the one BN-backward call whose apply launch takes both
    EmittedStats premerged;
    const float *premerged_stats = nullptr;
    int premerge_slot = 0;
    // Statistics from the producing epilogue: the driver lends a buffer
    // (emit_buf, emit_floats floats; null = off), conv_fwd sets want_emit for the
    // kernels it dispatches, a kernel that emits records what it described in
    // `emitted`, and the next bn_stats call consumes that record (match or not).
    float *emit_buf = nullptr;
    size_t emit_floats = 0;
    bool want_emit = false;
    EmittedStats emitted;
    hipStream_t stream = nullptr;
    bool dry = false;
    rvn_cost cost = {};
    hipError_t err = hipSuccess;
    hipEvent_t ev_start = nullptr, ev_stop = nullptr;  // set while a profiled launch is pending
    int last_id = 0;  // family of the latest launch(): a wrapper that needs further launches for the same
                      // operation (image slices of a tensor beyond 4 GB) records them under it, with no bytes

    // Record one kernel launch of family `id` that must move `bytes`
    // algorithmic bytes and perform `flops`; returns true if the kernel should
    // really be launched (then call run() for it).
    bool launch(int id, double bytes, double flops = 0.0) {
        last_id = id;
        cost.kernel_launches += 1;
        cost.algorithmic_bytes += bytes;
        const bool go = !dry && err == hipSuccess;
        if (go && profile_enabled()) profile_new_mark(id, bytes, flops, &ev_start, &ev_stop);
        return go;
    }
    // Enqueue `kernel` on the stream and record the launch status.  Counting mode enqueues nothing, so
    // that a wrapper whose later bookkeeping depends on what its dispatch decides (which kernel, what
    // it leaves for the next call) can walk through that dispatch when only counting.
    template <typename... KArgs, typename... Args>
    void run(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes, Args... args) {
        if (dry) return;
        if (ev_start) {
            hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, ev_start, ev_stop, 0,
                                  static_cast<KArgs>(args)...);
            ev_start = ev_stop = nullptr;
        } else {
            kernel<<<grid, block, lds_bytes, stream>>>(static_cast<KArgs>(args)...);
        }
        if (err == hipSuccess) err = hipGetLastError();
    }
    void fail(hipError_t e) {
        ev_start = ev_stop = nullptr;
        if (err == hipSuccess) err = e;
    }
};

// The second half of a filter gradient: the ordered sum of its partial results.
// conv_wgrad either launches it or hands it to the caller, who lets another
// launch carry it (bn_relu_bwd's apply pass).  blocks == 0: nothing to do.
struct WgradReduce {
    const float *part;  // [S][part_stride]
    float *dw;          // [CO][CI][KS2]
    int part_stride, S, KS2, MT, CT, tiles_c, CO, CI, accumulate;
    int tile;    // 16 (fp32 instruction) or 32 (bf16 instruction): edge of a result tile
    int wide;    // 1: one thread per slot sums all S slices (S small); 0: 8 threads share a slot
    int blocks;  // workgroups of 256 threads it needs
};

// ---- sizes of the small scratch areas the wrappers need (floats) ----------
// Number of image groups a per-channel reduction is split into.
int reduce_splits(int c, const Geo &g);
// Scratch floats for bn_stats / bn_relu_bwd partial results of `c` channels.
size_t bn_scratch_floats(int c, const Geo &g);
// Scratch floats for the filter-gradient partial sums.
size_t wgrad_scratch_floats(int cin, int cout, int ks, const Geo &g);
size_t wgrad_bf16_scratch_floats(int cin, int cout, int ks, const Geo &g);

// ---- batch norm + ReLU (Section 2.2: a(x) = ReLU(BN(x))) -------------------
// Per-channel statistics of x and the affine map they imply.  stats holds four
// arrays of c floats: batch mean, rstd = 1/sqrt(biased var + eps),
// scale = gamma*rstd, shift = beta - mean*scale, so that
// a(x) = max(x*scale + shift, 0).  Every consumer evaluates that one
// expression (one fma), which keeps the ReLU decisions of the forward pass, the
// recomputation and the backward pass identical.
constexpr int kStatsArrays = 4;
// `counters`: c * kCounterStride zero-initialised ints (ticket counters of the
// cross-workgroup reduction, one per channel, each on a cache line of its own
// so that the atomics of different channels do not serialise; left at zero
// again).
constexpr int kCounterStride = 32;
// `carry`: a filter conversion (see PrepArgs below) whose workgroups ride in this launch.
struct PrepArgs;
void bn_stats(Ctx &cx, View x, int c, Geo g, float eps, const float *gamma, const float *beta,
              float *scratch, int *counters, float *stats, const PrepArgs *carry = nullptr, double carry_bytes = 0.0);

// Zero n ticket counters (once per library call; the workspace is caller
// memory with unknown contents).
void clear_counters(Ctx &cx, int *counters, int n);

// Backward of a(x) given da (dense fp32): writes dgamma, dbeta (added to when
// accumulate) and out = [skip +] dx.  `skip` may be null.  `out` may alias
// `da` (dense in-place) or `skip`.  `carry`: a pending filter-gradient sum that
// rides in the apply launch (extra workgroups).
// out16 != null (needs h*w % 4 == 0 and 16-byte aligned x, da; no skip): the result goes there as
// dense bf16 [n][c][h*w], rounded to nearest even, and `out` is not written; out16 must not overlap da.
void bn_relu_bwd(Ctx &cx, View x, const float *da, int c, Geo g, const float *stats, float *scratch,
                 int *counters, float *dgamma, float *dbeta, bool accumulate, const View *skip, View out,
                 const WgradReduce *carry = nullptr, uint16_t *out16 = nullptr);

// ---- convolutions (Section 2.2: c_k(x) = Conv_kxk(a(x)), k in {1,3}) -------
// out = ep(r, conv(a(x), w)) with a(x) = max(x*scale + shift, 0) formed on the
// fly from stats (scale_shift = stats + 2*cin); w is fp32 [cout][cin][ks][ks].
// With dt == RVN_BF16 both operands are rounded to bf16 before multiplying.
void conv_fwd(Ctx &cx, View x, const float *scale_shift, rvn_dtype dt, const float *w, const uint16_t *wq, int cin,
              int cout, int ks, Geo g, Epilogue ep, const View *r, View out, float *scratch);

// The same convolution on bf16 matrix instructions (operands rounded to bf16,
// fp32 accumulation); `transposed`: w is [ci][co][ks][ks] and is read transposed
// and flipped (data gradient).  Returns false if no tiling fits (nothing is
// launched then).
bool conv_bf16(Ctx &cx, View in, const float *scale_shift, const float *w, const uint16_t *wq, bool transposed,
               int ci, int co, int ks, Geo g, Epilogue ep, const View *r, View out, float *scratch);
// Scratch floats conv_bf16 may need for a ci -> co convolution (partial tiles
// when the input channels are split over workgroups); 0 if none.
size_t conv_bf16_scratch_floats(int ci, int co, int ks, const Geo &g);

// 3x3 convolution, register-tiled and software-pipelined (see conv3x3_bf16.hip).
// Needs the filter prepared as [co][9][ci padded to 8]; returns false (nothing
// launched) when conv3x3_bf16_ok(ci, co, g) does not hold.
bool conv3x3_bf16_ok(int ci, int co, const Geo &g);
size_t conv3x3_bf16_scratch_floats(int ci, int co, const Geo &g, int stride = 1);
// The 3x3 convolution with stride 2 (g: the input's geometry, h and w even; out: [n][co][h/2][w/2], store only),
// accounted as a forward convolution; false (nothing launched, nothing accounted) if the kernel does not take it.
bool conv3x3_bf16_stride2(Ctx &cx, View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g, View out,
                          float *scratch);
bool conv3x3_bf16(Ctx &cx, View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g,
                  Epilogue ep, const View *r, View out, float *scratch);

PrepArgs plan_filter_prep(const FilterPrep *f, int count, Geo g, double *bytes);
void prep_filters_bf16(Ctx &cx, const PrepArgs &a, double bytes);

// 1x1 convolution without LDS: activations go from HBM to the matrix
// instruction's registers directly.  Needs the filter in operand order (wq from
// prep_filters_bf16) and conv1x1_direct_ok(ci, g); returns false (nothing
// launched) otherwise.
bool conv1x1_direct_ok(int k_channels, const Geo &g);
size_t filter_1x1_elems(int rows, int k_channels);
bool conv1x1_bf16(Ctx &cx, View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g,
                  Epilogue ep, const View *r, View out);

// da (dense fp32 [n][cin][h*w]) = sum_{k,r,s} dh[.., k, p-r+pad, q-s+pad] w[k,c,r,s];
// dh is fp32, rounded to bf16 on load when dt == RVN_BF16.
void conv_dgrad(Ctx &cx, View dh, rvn_dtype dt, const float *w, const uint16_t *wq, int cin, int cout, int ks,
                Geo g, float *da, float *scratch);

// dw[k,c,r,s] (+)= sum_{n,p,q} dh[n,k,p,q] a[n,c,p+r-pad,q+s-pad], with
// a(x) = max(x*scale + shift, 0) formed on the fly from the layer input x as in
// conv_fwd; with dt == RVN_BF16 a and dh are rounded to bf16 before multiplying.
// With `defer` the ordered sum of the partial results is not launched but
// described in *defer for the caller to run (before `scratch` is reused).
void conv_wgrad(Ctx &cx, View x, const float *scale_shift, rvn_dtype dt, View dh, int cin, int cout,
                int ks, Geo g, float *scratch, float *dw, bool accumulate, WgradReduce *defer = nullptr);
void wgrad_reduce(Ctx &cx, const WgradReduce &r);

// True while the environment variable RVN_SEPARATE_LAUNCHES is "1": the data gradient and the filter
// gradient of a layer then always get a launch each (a diagnostic switch, read at every call; the
// results do not depend on it, bit for bit).
bool separate_launches();

// conv_dgrad and conv_wgrad of one fp32 3x3 layer in a single launch (both need
// only dh); the ordered sum of the filter gradient is left in *defer.  Returns
// false (nothing launched, nothing accounted) for the shapes it does not take.
bool conv_dgrad_wgrad_f32(Ctx &cx, View x, const float *scale_shift, View dh, const float *w, int cin, int cout,
                          int ks, Geo g, float *scratch, float *dw, bool accumulate, float *da, WgradReduce *defer);

// conv_dgrad and conv_wgrad of one layer with bf16 operands (1x1 or 3x3) in a single launch; wq_b is the
// filter prepared for the data gradient.  The ordered sum of the filter gradient is left in *defer; a
// channel-split data gradient is followed by its reduce launch.  Returns false (nothing launched,
// nothing accounted) for the shapes it does not take.
// dh16 != null: the upstream gradient is there as dense bf16 [n][cout][h*w] (what rounding dh on load
// would give, so the results are the same bits) and `dh` is ignored; only for layers for which
// conv_dgrad_wgrad_takes_bf16_dh says yes.
bool conv_dgrad_wgrad_bf16(Ctx &cx, View x, const float *scale_shift, View dh, const uint16_t *dh16, const uint16_t *wq_b,
                           int cin, int cout, int ks, Geo g, float *wgrad_scratch, float *dw, bool accumulate,
                           float *da, float *conv_scratch, WgradReduce *defer);
bool conv_dgrad_wgrad_takes_bf16_dh(View x, const uint16_t *dh16, const uint16_t *wq_b, int cin, int cout, int ks, Geo g,
                                    float *wgrad_scratch, float *da, float *conv_scratch);

// The filter gradient with bf16 operands on v_mfma_f32_32x32x16_bf16 (a(x) and dh rounded
// to bf16 while staged, fp32 accumulation); `bytes` and `flops` are what the
// caller accounts for the launch.  Returns false (nothing launched) when no
// plan fits; scratch must hold wgrad_bf16_scratch_floats(...) floats.
bool conv_wgrad_bf16(Ctx &cx, View x, const float *scale_shift, View dh, int cin, int cout, int ks, Geo g,
                     float *scratch, float *dw, bool accumulate, double bytes, double flops, WgradReduce *defer);

// ---- fixed-point residual stream (Section 3.2, "Numerical error") ------------
// A stream element is an int32 code q standing for q * 2^-frac_bits; the Views
// of stream tensors carry int32 data behind their float pointer.
// out (dense fp32 [n][c][h*w]) = float(x) * 2^-frac_bits.
void fix_to_float(Ctx &cx, View x, int c, Geo g, int frac_bits, float *out);
// out = r + sign * rint(f * 2^frac_bits) as an integer sum; f dense fp32, sign = +1 or -1; out may be r.
void fix_axpy(Ctx &cx, View r, const float *f, int c, Geo g, int frac_bits, int sign, View out);
// out (int32 codes) = rint(x * 2^frac_bits).
void fix_from_float(Ctx &cx, View x, int c, Geo g, int frac_bits, View out);

// ---- stem: image convolution and max-pooling ahead of the reversible stages ----
// Direct fp32 kernels for a convolution whose input has a handful of channels
// (c_in * k * k <= 256), stride 1 or 2, padding (k-1)/2; HO, WO are its output size.
struct StemShape {
    int N, CI, H, W, CO, KS, stride, HO, WO;
};
void stem_conv(Ctx &cx, View x, const float *w, const StemShape &g, View out);
// The same on the matrix cores (stem_mfma.hip) for the shapes it takes; stem_conv dispatches.
bool stem_conv_mfma_takes(const StemShape &g);
void stem_conv_mfma(Ctx &cx, View x, const float *w, const StemShape &g, View out);
// Filter gradient on the matrix cores: partial results part[chunk][k][tap] for stem_wgrad's reduce pass;
// stem_wgrad_mfma_chunks is 0 for shapes it does not take.
int stem_wgrad_mfma_chunks(const StemShape &g);
void stem_wgrad_mfma(Ctx &cx, View x, View dh, const StemShape &g, float *part);
// dw[k][c][r][s] (+)= sum over output pixels of dh * x; scratch: stem_wgrad_scratch_floats(g) floats.
size_t stem_wgrad_scratch_floats(const StemShape &g);
void stem_wgrad(Ctx &cx, View x, View dh, const StemShape &g, float *scratch, float *dw, bool accumulate);
// 3x3 windows, stride 2, padding 1 (outside positions never win); output size ((h-1)/2+1, (w-1)/2+1).
// The derivative of a window goes to its first maximal element in row-major order.
void maxpool3s2_fwd(Ctx &cx, View x, int c, Geo in, View y);
// dx dense [n][c][h][w]; scratch: maxpool3s2_scratch_bytes(c, in) bytes (the windows' winners).
size_t maxpool3s2_scratch_bytes(int c, Geo in);
void maxpool3s2_bwd(Ctx &cx, View x, View dy, int c, Geo in, unsigned char *scratch, float *dx);

// ---- stride-2 resampling for the non-reversible subsampling block ----------
// `full` is the geometry of the high-resolution side (h, w even).
// out (dense [n][c][h/2][w/2]) = every second row and column of `in`.
void subsample2(Ctx &cx, View in, int c, Geo full, float *out);
// out (dense [n][c][h][w]) = `in` (dense, half resolution) at the even positions, zero elsewhere.
void upsample2_zero(Ctx &cx, const float *in, int c, Geo full, float *out);
// acc (dense [n][c][h][w]) += t (dense, half resolution) at the even positions.
void upsample2_add(Ctx &cx, const float *t, int c, Geo full, float *acc);

}  // namespace rvn
