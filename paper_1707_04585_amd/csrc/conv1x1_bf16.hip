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
#include <type_traits>

#include "kernels.h"
#include "stats_fold.h"

namespace rvn {

namespace {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef float f4a_t __attribute__((ext_vector_type(4)));              // 16-byte aligned
typedef float f4u_t __attribute__((ext_vector_type(4), aligned(4)));  // only element aligned
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

struct C1Args {
    const float *in;  // x (forward) or upstream gradient (data gradient), fp32, planes of HW floats
    int64_t isn, isc;
    const float *scale_shift;  // [2*CI]: a = max(in*scale + shift, 0); null = use `in` as is
    const uint16_t *wq;        // filter in operand order: [mtiles][ksteps][64 lanes][8]
    const float *r;            // skip operand of the epilogue (may alias out)
    int64_t rsn, rsc;
    float *out;
    int64_t osn, osc;
    int HW, CI, CO;
    int ep;
    int gpi, groups;  // 4-pixel groups per image and in total
    int ksteps;       // CI / 16
    int mtiles;       // ceil(CO / 32)
    float *emit;      // per (channel, 128-pixel tile) mean and M2 of the output (EMIT variants; needs whole tiles)
    int ptiles;       // pixel tiles in all
    int PW, CW, KW;   // wavefronts of a workgroup: pixel tiles x output-channel tiles x shares of the channels
    int npt, ncg;     // workgroup grid: pixel tiles / PW, output-channel tiles / CW
    uint32_t m_gpi;   // fast-division multiplier (see fdiv)
};

__device__ __forceinline__ int fdiv(int e, uint32_t m) { return m ? (int)__umulhi((uint32_t)e, m) : e; }

// Two floats to a pair of bf16 (nearest even): one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const float2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<const uint32_t *>(&b);
}

// MTW: 32-channel output tiles per wavefront.  DEPTH: steps the loads run ahead
// (1 or 2).  GEN: planes need not be 16-byte
// aligned and H*W need not be a multiple of 4 (the last group of an image then
// starts at H*W - 4 and leaves the pixels it shares with its neighbour to it).
template <int MTW, int DEPTH, bool GEN, bool EMIT = false>
__global__ __launch_bounds__(kThreads, 2) void conv1x1_bf16_k(const C1Args p) {
    using F4 = typename std::conditional<GEN, f4u_t, f4a_t>::type;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, kg = lane >> 5;

    // Workgroup ids go round-robin over the 8 dies; give every die a contiguous
    // range of the (pixel tile, channel tile) space so that workgroups sharing
    // input data also share an L2.
    const int per_die = gridDim.x >> 3;
    const int logical = (blockIdx.x & 7) * per_die + (blockIdx.x >> 3);
    const int cg = logical % p.ncg, pt = logical / p.ncg;
    if (pt >= p.npt) return;
    const int pw = wave % p.PW, cw = (wave / p.PW) % p.CW, kw = wave / (p.PW * p.CW);
    const int mt0 = (cg * p.CW + cw) * MTW;
    const bool idle = mt0 >= p.mtiles;  // no output tile: only keeps the barrier company

    const int HW = p.HW;
    const int g = (pt * p.PW + pw) * 32 + l32;
    const bool live = g < p.groups;
    const int gg = live ? g : 0;
    const int n = fdiv(gg, p.m_gpi), q = gg - n * p.gpi;
    // The last group of an image may have fewer than 4 pixels left (GEN): its
    // window is moved back so that it ends with the plane, pix = H*W - 4.  Its first
    // `dup` pixels then repeat the previous group's (computed again, not stored),
    // so no data has to be shifted or masked on the way to the matrix instructions.
    const int dup = GEN ? max(0, 4 * q + 4 - HW) : 0;
    const int pix = 4 * q - dup;
    // Addresses are a wavefront-uniform 64-bit part (channel, step) plus a 32-bit
    // per-lane byte offset (image, pixel, channel octet half): the host keeps
    // every tensor slice handed to one launch below 4 GB.
    const uint32_t in_off = (uint32_t)(((int64_t)n * p.isn + pix + (int64_t)(kg * 8) * p.isc) * 4);
    const char *const in_base = reinterpret_cast<const char *>(p.in);
    const int64_t isc_b = p.isc * 4;
    const char *const w_base = reinterpret_cast<const char *>(p.wq) + (int64_t)mt0 * p.ksteps * 1024;
    const uint32_t w_off = (uint32_t)lane * 16;
    const int64_t tile_w = (int64_t)p.ksteps * 1024;
    const bool bn = p.scale_shift != nullptr;
    const int CI = p.CI;

    // Output addressing: uniform 64-bit channel part plus a 32-bit lane offset.
    const uint32_t o_off = (uint32_t)(((int64_t)n * p.osn + pix + (int64_t)(4 * kg) * p.osc) * 4);
    const uint32_t r_off = (uint32_t)(((int64_t)n * p.rsn + pix + (int64_t)(4 * kg) * p.rsc) * 4);
    char *const o_base = reinterpret_cast<char *>(p.out);
    const char *const r_base = reinterpret_cast<const char *>(p.r);
    // channel of register i of output tile m, without the lane's 4*kg
    auto chan = [&](int m, int i) { return (mt0 + m) * 32 + 8 * (i >> 2) + (i & 3); };

    // The accumulators start from the skip operand (+r for y = r + conv, -r for
    // x = r - conv, negated again when stored), so its loads are in flight
    // together with the first activation loads and cost no registers.  r may
    // alias out element for element: a lane reads an address before it writes it.
    // The loads are unconditional (a lane with nothing to fetch re-reads its own first valid address, or
    // the tensor base, and the value is discarded afterwards): a load inside a divergent branch makes the
    // compiler wait for it before the next one is issued, one memory round trip per register.
    float16_t acc[MTW][4];
    if (p.ep != EP_STORE) {
        const bool fetch = live && !idle && kw == 0;
        const float sign = p.ep == EP_SUB ? -1.f : 1.f;
        F4 t[MTW][16];
#pragma unroll
        for (int m = 0; m < MTW; ++m)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const bool ok = fetch && chan(m, i) + 4 * kg < p.CO;
                const int64_t off = ok ? (int64_t)chan(m, i) * p.rsc * 4 + r_off : 0;
                t[m][i] = *reinterpret_cast<const F4 *>(r_base + off);
            }
#pragma unroll
        for (int m = 0; m < MTW; ++m)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const bool ok = fetch && chan(m, i) + 4 * kg < p.CO;
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[m][j][i] = ok ? sign * t[m][i][j] : 0.f;
            }
    } else {
#pragma unroll
        for (int m = 0; m < MTW; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[m][j][i] = 0.f;
    }

    struct Buf {
        F4 v[8];
        uint4_t a[MTW];
    };
    auto load = [&](Buf &b, int ks) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            b.v[k] = *reinterpret_cast<const F4 *>(in_base + (int64_t)(ks * 16 + k) * isc_b + in_off);
#pragma unroll
        for (int m = 0; m < MTW; ++m) {
            const bool has = mt0 + m < p.mtiles;
            b.a[m] = *reinterpret_cast<const uint4_t *>(w_base + (has ? m * tile_w : 0) + (int64_t)ks * 1024 + w_off);
        }
    };
    auto compute = [&](Buf &b, int ks) {
        float v[8][4];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            float x0 = b.v[k][0], x1 = b.v[k][1], x2 = b.v[k][2], x3 = b.v[k][3];
            if (bn) {
                const int c = ks * 16 + k;  // wavefront-uniform: scalar loads
                const float s_lo = p.scale_shift[c], s_hi = p.scale_shift[c + 8];
                const float h_lo = p.scale_shift[CI + c], h_hi = p.scale_shift[CI + c + 8];
                const float sc = kg ? s_hi : s_lo, sh = kg ? h_hi : h_lo;
                x0 = fmaxf(fmaf(x0, sc, sh), 0.f);
                x1 = fmaxf(fmaf(x1, sc, sh), 0.f);
                x2 = fmaxf(fmaf(x2, sc, sh), 0.f);
                x3 = fmaxf(fmaf(x3, sc, sh), 0.f);
            }
            v[k][0] = x0; v[k][1] = x1; v[k][2] = x2; v[k][3] = x3;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint4_t bq = {pack2(v[0][j], v[1][j]), pack2(v[2][j], v[3][j]), pack2(v[4][j], v[5][j]),
                                pack2(v[6][j], v[7][j])};
            const bf16x8_t bo = *reinterpret_cast<const bf16x8_t *>(&bq);
#pragma unroll
            for (int m = 0; m < MTW; ++m)
                acc[m][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t *>(&b.a[m]), bo,
                                                                    acc[m][j], 0, 0, 0);
        }
    };

    // This wavefront's share of the reduction (KW wavefronts split the channels);
    // loads run DEPTH steps ahead of the arithmetic.
    const int ks0 = idle ? 0 : kw * p.ksteps / p.KW;
    const int ksteps = idle ? 0 : (kw + 1) * p.ksteps / p.KW;
    if (DEPTH == 1) {
        Buf b0, b1;
        if (ks0 < ksteps) load(b0, ks0);
        for (int ks = ks0; ks < ksteps; ks += 2) {
            if (ks + 1 < ksteps) load(b1, ks + 1);
            compute(b0, ks);
            if (ks + 1 < ksteps) {
                if (ks + 2 < ksteps) load(b0, ks + 2);
                compute(b1, ks + 1);
            }
        }
    } else {
        Buf b0, b1, b2;
        if (ks0 < ksteps) load(b0, ks0);
        if (ks0 + 1 < ksteps) load(b1, ks0 + 1);
        for (int ks = ks0; ks < ksteps; ks += 3) {
            if (ks + 2 < ksteps) load(b2, ks + 2);
            compute(b0, ks);
            if (ks + 1 < ksteps) {
                if (ks + 3 < ksteps) load(b0, ks + 3);
                compute(b1, ks + 1);
            }
            if (ks + 2 < ksteps) {
                if (ks + 4 < ksteps) load(b1, ks + 4);
                compute(b2, ks + 2);
            }
        }
    }

    // ---- epilogue: register i of accumulator (m, j) is channel
    //      (mt0 + m)*32 + 8*(i/4) + 4*kg + i%4 at pixel pix + j
    if (p.KW > 1) {  // sum the KW partial tiles in wavefront kw = 0, in a fixed order
        extern __shared__ float red[];  // [KW - 1][PW * CW][MTW * 64 registers][64 lanes]
        const int slot = wave % (p.PW * p.CW), slots = p.PW * p.CW;
        if (kw > 0) {
            float *dst = red + ((int64_t)((kw - 1) * slots + slot) * (MTW * 64)) * 64 + lane;
#pragma unroll
            for (int m = 0; m < MTW; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 16; ++i) dst[((m * 4 + j) * 16 + i) * 64] = acc[m][j][i];
        }
        __syncthreads();
        if (kw > 0) return;
        for (int k = 1; k < p.KW; ++k) {
            const float *srcp = red + ((int64_t)((k - 1) * slots + slot) * (MTW * 64)) * 64 + lane;
#pragma unroll
            for (int m = 0; m < MTW; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[m][j][i] += srcp[((m * 4 + j) * 16 + i) * 64];
        }
    }
    if (!live || idle) return;
    // Statistics of the stored values for the BN layer that reads them next
    // (host: aligned variant, every tile whole): a channel's 128 pixels
    // of this tile sit in the 32 lanes of one half, 4 per lane.  Sums of
    // (v - pivot) and (v - pivot)^2, pivot = the half's first value, are folded
    // over the lanes 16 channels at a time: each step halves the channels a lane
    // holds and adds its partner's, so 16 + 16 shuffles do all of them and every
    // sum has a fixed order.
    constexpr bool emit = EMIT && !GEN;
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
        float ea[16], eb[16], piv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            ea[i] = eb[i] = piv[i] = 0.f;
            if (chan(m, i) + 4 * kg >= p.CO) continue;
            F4 t = {acc[m][0][i], acc[m][1][i], acc[m][2][i], acc[m][3][i]};
            if (p.ep == EP_SUB) t = -t;
            float *op = reinterpret_cast<float *>(o_base + (int64_t)chan(m, i) * p.osc * 4 + o_off);
            if (!GEN || dup == 0) {
                *reinterpret_cast<F4 *>(op) = t;
            } else {  // the first dup pixels belong to the previous group
                if (dup < 2) op[1] = t[1];
                if (dup < 3) op[2] = t[2];
                op[3] = t[3];
            }
            if constexpr (emit) {
                const int t0 = __float_as_int(t[0]);
                const float lo = __int_as_float(__builtin_amdgcn_readlane(t0, 0));
                const float hi = __int_as_float(__builtin_amdgcn_readlane(t0, 32));
                piv[i] = kg ? hi : lo;
                const float d0 = t[0] - piv[i], d1 = t[1] - piv[i], d2 = t[2] - piv[i], d3 = t[3] - piv[i];
                ea[i] = (d0 + d1) + (d2 + d3);
                eb[i] = (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
            }
        }
        if constexpr (emit) {
            fold_16_channels(ea, eb, piv, l32);
            // the lane now holds register i = l32 / 2 of this tile
            const int i = l32 >> 1;
            const int c = (mt0 + m) * 32 + 8 * (i >> 2) + 4 * kg + (i & 3);
            if ((l32 & 1) == 0 && c < p.CO) {
                const float mean = piv[0] + ea[0] * (1.f / 128.f);
                const float m2 = fmaxf(eb[0] - ea[0] * ea[0] * (1.f / 128.f), 0.f);
                float2 *dst = reinterpret_cast<float2 *>(p.emit) + (int64_t)c * p.ptiles + (pt * p.PW + pw);
                *dst = make_float2(mean, m2);
            }
        }
    }
}

uint32_t fdiv_magic(int d) { return d == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)d + 1ull); }

size_t operand_elems(int rows, int cols) { return (size_t)((rows + 31) / 32) * 32 * ((cols + 15) / 16) * 16; }

}  // namespace

bool conv1x1_direct_ok(int k_channels, const Geo &g) {
    return k_channels % 16 == 0 && (int64_t)g.h * g.w >= 4 && (int64_t)g.n * ((g.h * g.w + 3) / 4) < (1 << 30);
}

size_t filter_1x1_elems(int rows, int k_channels) { return operand_elems(rows, k_channels); }

bool conv1x1_bf16(Ctx &cx, View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g,
                  Epilogue ep, const View *r, View out) {
    if (!wq || !conv1x1_direct_ok(ci, g)) return false;
    const int HW = g.h * g.w;
    // Lane offsets are 32-bit byte offsets from the tensor base: launch per slice
    // of images small enough for that.
    const int64_t img_bytes = 4 * std::max(std::max(in.sn, out.sn), r ? r->sn : (int64_t)0);
    const int64_t tail_bytes = 4 * ((int64_t)HW + std::max(std::max((int64_t)ci * in.sc, (int64_t)co * out.sc),
                                                           r ? (int64_t)co * r->sc : (int64_t)0));
    const int64_t room = ((int64_t)1 << 32) - tail_bytes;
    if (room < img_bytes) {  // one image alone is too large
        cx.fail(hipErrorInvalidValue);
        return true;
    }
    const int slice_n = (int)std::min<int64_t>(g.n, room / std::max<int64_t>(img_bytes, 1));
    for (int n0 = 0; n0 < g.n; n0 += slice_n) {
        const int ns = std::min(slice_n, g.n - n0);
        C1Args a{};
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
        int mtw = a.KW == 1 && a.mtiles >= 2 && (int64_t)ptiles * ((a.mtiles + 1) / 2) >= 1024 ? 2 : 1;
        const int cot = (a.mtiles + mtw - 1) / mtw;
        const int rest = 4 / a.KW;
        a.CW = cot >= rest ? rest : cot >= 2 ? 2 : 1;
        a.PW = rest / a.CW;
        a.npt = (ptiles + a.PW - 1) / a.PW;
        a.ncg = (cot + a.CW - 1) / a.CW;
        const int64_t wgs = ((int64_t)a.npt * a.ncg + 7) / 8 * 8;
        const bool gen = (HW & 3) != 0 || (in.sn & 3) != 0 || (in.sc & 3) != 0 || (out.sn & 3) != 0 ||
                         (out.sc & 3) != 0 || (reinterpret_cast<uintptr_t>(in.p) & 15) != 0 ||
                         (reinterpret_cast<uintptr_t>(out.p) & 15) != 0 ||
                         (r && ((r->sn & 3) != 0 || (r->sc & 3) != 0 || (reinterpret_cast<uintptr_t>(r->p) & 15) != 0));
        // Statistics of the output for the BN layer that reads it next: whole 128-pixel tiles, aligned
        // variant, one launch for all images (with channel shares the wavefront holding the final sums emits).
        const bool emits = cx.want_emit && cx.emit_buf && !gen && a.groups % 32 == 0 && ns == g.n &&
                           (size_t)co * ptiles * 2 <= cx.emit_floats;
        a.emit = emits ? cx.emit_buf : nullptr;
        if (emits) cx.emitted = EmittedStats{out.p, out.sn, out.sc, co, g.n, g.h, g.w, ptiles, 128};
        const dim3 grid((unsigned)wgs);
        const size_t lds = a.KW > 1 ? (size_t)(a.KW - 1) * (a.PW * a.CW) * mtw * 64 * 64 * 4 : 0;
        const int depth = mtw == 1 ? 2 : 1;
        if (emits) {  // (never the general variant)
            if (mtw == 2) cx.run(conv1x1_bf16_k<2, 1, false, true>, grid, dim3(kThreads), lds, a);
            else if (depth == 2) cx.run(conv1x1_bf16_k<1, 2, false, true>, grid, dim3(kThreads), lds, a);
            else cx.run(conv1x1_bf16_k<1, 1, false, true>, grid, dim3(kThreads), lds, a);
        } else if (mtw == 2) {
            if (gen) cx.run(conv1x1_bf16_k<2, 1, true>, grid, dim3(kThreads), lds, a);
            else cx.run(conv1x1_bf16_k<2, 1, false>, grid, dim3(kThreads), lds, a);
        } else if (depth == 2) {
            if (gen) cx.run(conv1x1_bf16_k<1, 2, true>, grid, dim3(kThreads), lds, a);
            else cx.run(conv1x1_bf16_k<1, 2, false>, grid, dim3(kThreads), lds, a);
        } else {
            if (gen) cx.run(conv1x1_bf16_k<1, 1, true>, grid, dim3(kThreads), lds, a);
            else cx.run(conv1x1_bf16_k<1, 1, false>, grid, dim3(kThreads), lds, a);
        }
    }
    return true;
}

}  // namespace rvn
