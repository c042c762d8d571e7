// 1x1 convolution (forward and data gradient) with bf16 operands on the CDNA4
// matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation), for the 1x1 units
// of the bottleneck residual function (Section 2.2, Eq. 3) when the block
// descriptor asks for bf16 convolution operands.
//
// A 1x1 convolution has no halo, so the activation operand never needs LDS: the
// image plane of a channel is a contiguous run of H*W floats, and a lane loads
// 4 consecutive pixels of 8 consecutive channels (8 coalesced 16-byte loads per
// 16-channel step).  Element j of those loads, over the 8 channels, is exactly
// the B operand of one matrix instruction for the lane's pixel 4*q + j, so a
// wavefront covers 32 groups of 4 pixels with 4 matrix instructions per step
// and its results come out as 4 consecutive pixels per lane and channel:
// 16-byte stores, 512-byte runs per channel.  BN scale/shift, ReLU and the bf16
// rounding are applied in registers between the load and the multiply; the
// coupling y = r + acc / reconstruction x = r - acc of Section 3.1 is applied in
// the accumulator registers.
//
// The filter is read from a copy laid out in operand order (one contiguous
// 1 KB block per 32 output channels x 16 input channels, lane-major), so the A
// operand is a single coalesced 16-byte load per lane that stays in L1/L2.
// The loads of step s+1 are issued before the arithmetic of step s.  There is
// no LDS and no barrier: the four wavefronts of a workgroup are independent
// and are arranged as PW pixel tiles x CW output-channel tiles so that those
// which share input data run on the same compute unit.
#include <algorithm>

#include "conv1x1_bf16_body.h"
#include "kernels.h"

namespace rvn {

namespace {

using namespace c1;

template <int MTW, int DEPTH, bool GEN, bool EMIT = false>
__global__ __launch_bounds__(kThreads, 2) void conv1x1_bf16_k(const C1Args p) {
    extern __shared__ float red[];
    conv1x1_bf16_body<MTW, DEPTH, GEN, EMIT>(p, blockIdx.x, gridDim.x, red);
}

uint32_t fdiv_magic(int d) { return d == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)d + 1ull); }

size_t operand_elems(int rows, int cols) { return (size_t)((rows + 31) / 32) * 32 * ((cols + 15) / 16) * 16; }

}  // namespace

bool conv1x1_direct_ok(int k_channels, const Geo &g) {
    return k_channels % 16 == 0 && (int64_t)g.h * g.w >= 4 && (int64_t)g.n * ((g.h * g.w + 3) / 4) < (1 << 30);
}

size_t filter_1x1_elems(int rows, int k_channels) { return operand_elems(rows, k_channels); }

namespace {

// Arguments and tiling for the images [n0, n0 + ns) of the tensors.
C1Launch plan_slice(View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g, Epilogue ep,
                    const View *r, View out, int n0, int ns) {
    const int HW = g.h * g.w;
    C1Launch L{};
    C1Args &a = L.a;
    a.in = in.p + (int64_t)n0 * in.sn; a.isn = in.sn; a.isc = in.sc;
    a.scale_shift = scale_shift;
    a.wq = wq;
    a.r = r ? r->p + (int64_t)n0 * r->sn : nullptr; a.rsn = r ? r->sn : 0; a.rsc = r ? r->sc : 0;
    a.out = out.p + (int64_t)n0 * out.sn; a.osn = out.sn; a.osc = out.sc;
    a.HW = HW; a.CI = ci; a.CO = co;
    a.ep = (int)ep;
    a.gpi = (HW + 3) / 4;
    a.groups = ns * a.gpi;
    a.ksteps = ci / 16;
    a.mtiles = (co + 31) / 32;
    a.m_gpi = fdiv_magic(a.gpi);
    const int ptiles = (a.groups + 31) / 32;
    a.ptiles = ptiles;
    // With few tiles, the wavefronts of a workgroup split the input channels
    // (shorter dependent chains, more loads in flight).  Otherwise two output
    // tiles per wavefront halve the passes over the input, once the halved
    // tile count still fills the chip four times over.
    const int64_t tiles = (int64_t)ptiles * a.mtiles;
    a.KW = 1;
    if (tiles < 1024 && a.ksteps >= 8) a.KW = tiles < 512 && a.ksteps >= 16 ? 4 : 2;
    // (1024 wavefront tiles: at the 56x56 bottleneck layers two tiles per wavefront took 5-13 % off the
    // launch, at 28x28 -- 784 tiles left -- they cost 3 %)
    L.mtw = a.KW == 1 && a.mtiles >= 2 && (int64_t)ptiles * ((a.mtiles + 1) / 2) >= 1024 ? 2 : 1;
    L.depth = L.mtw == 1 ? 2 : 1;
    const int cot = (a.mtiles + L.mtw - 1) / L.mtw;
    const int rest = 4 / a.KW;
    a.CW = cot >= rest ? rest : cot >= 2 ? 2 : 1;
    a.PW = rest / a.CW;
    a.npt = (ptiles + a.PW - 1) / a.PW;
    a.ncg = (cot + a.CW - 1) / a.CW;
    L.wgs = (unsigned)(((int64_t)a.npt * a.ncg + 7) / 8 * 8);
    L.gen = (HW & 3) != 0 || (in.sn & 3) != 0 || (in.sc & 3) != 0 || (out.sn & 3) != 0 || (out.sc & 3) != 0 ||
            (reinterpret_cast<uintptr_t>(in.p) & 15) != 0 || (reinterpret_cast<uintptr_t>(out.p) & 15) != 0 ||
            (r && ((r->sn & 3) != 0 || (r->sc & 3) != 0 || (reinterpret_cast<uintptr_t>(r->p) & 15) != 0));
    L.lds_bytes = a.KW > 1 ? (size_t)(a.KW - 1) * (a.PW * a.CW) * L.mtw * 64 * 64 * 4 : 0;
    return L;
}

// Lane offsets are 32-bit byte offsets from the tensor base: the images one launch can take (0: one
// image alone is too large).
int images_per_launch(View in, const View *r, View out, int ci, int co, Geo g) {
    const int64_t img_bytes = 4 * std::max(std::max(in.sn, out.sn), r ? r->sn : (int64_t)0);
    const int64_t tail_bytes = 4 * ((int64_t)g.h * g.w + std::max(std::max((int64_t)ci * in.sc, (int64_t)co * out.sc),
                                                                  r ? (int64_t)co * r->sc : (int64_t)0));
    const int64_t room = ((int64_t)1 << 32) - tail_bytes;
    if (room < img_bytes) return 0;
    return (int)std::min<int64_t>(g.n, room / std::max<int64_t>(img_bytes, 1));
}

}  // namespace

bool conv1x1_bf16_plan(View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g, Epilogue ep,
                       const View *r, View out, C1Launch &L) {
    if (!wq || !conv1x1_direct_ok(ci, g) || images_per_launch(in, r, out, ci, co, g) < g.n) return false;
    L = plan_slice(in, scale_shift, wq, ci, co, g, ep, r, out, 0, g.n);
    return true;
}

bool conv1x1_bf16(Ctx &cx, View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g,
                  Epilogue ep, const View *r, View out) {
    if (!wq || !conv1x1_direct_ok(ci, g)) return false;
    const int slice_n = images_per_launch(in, r, out, ci, co, g);
    if (slice_n == 0) {  // one image alone is too large
        cx.fail(hipErrorInvalidValue);
        return true;
    }
    for (int n0 = 0; n0 < g.n; n0 += slice_n) {
        const int ns = std::min(slice_n, g.n - n0);
        // (the caller has recorded the first launch; further slices are launches of the same family, their
        // bytes and flops already counted with the first)
        if (n0 > 0 && !cx.launch(cx.last_id, 0.0) && !cx.dry) return true;
        C1Launch L = plan_slice(in, scale_shift, wq, ci, co, g, ep, r, out, n0, ns);
        C1Args &a = L.a;
        // Statistics of the output for the BN layer that reads it next: whole 128-pixel tiles, aligned
        // variant, one launch for all images (with channel shares the wavefront holding the final sums emits).
        const bool emits = cx.want_emit && cx.emit_buf && !L.gen && a.groups % 32 == 0 && ns == g.n &&
                           (size_t)co * a.ptiles * 2 <= cx.emit_floats;
        a.emit = emits ? cx.emit_buf : nullptr;
        if (emits) cx.emitted = EmittedStats{out.p, out.sn, out.sc, co, g.n, g.h, g.w, a.ptiles, 128};
        const dim3 grid(L.wgs);
        if (emits) {  // (never the general variant)
            if (L.mtw == 2) cx.run(conv1x1_bf16_k<2, 1, false, true>, grid, dim3(kThreads), L.lds_bytes, a);
            else cx.run(conv1x1_bf16_k<1, 2, false, true>, grid, dim3(kThreads), L.lds_bytes, a);
        } else if (L.mtw == 2) {
            if (L.gen) cx.run(conv1x1_bf16_k<2, 1, true>, grid, dim3(kThreads), L.lds_bytes, a);
            else cx.run(conv1x1_bf16_k<2, 1, false>, grid, dim3(kThreads), L.lds_bytes, a);
        } else {
            if (L.gen) cx.run(conv1x1_bf16_k<1, 2, true>, grid, dim3(kThreads), L.lds_bytes, a);
            else cx.run(conv1x1_bf16_k<1, 2, false>, grid, dim3(kThreads), L.lds_bytes, a);
        }
    }
    return true;
}

}  // namespace rvn
