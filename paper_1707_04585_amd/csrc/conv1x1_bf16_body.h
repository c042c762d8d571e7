// Kernel body and argument block of the 1x1 convolution with bf16 operands (see
// conv1x1_bf16.hip for the design), as a device function so that a launch can
// hold it next to another body.  Device code only.
#pragma once

#include <type_traits>

#include "kernels.h"
#include "stats_fold.h"

namespace rvn {

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

// What a launch of the convolution needs besides its arguments.
struct C1Launch {
    C1Args a;
    int mtw, depth;  // output tiles per wavefront, steps the loads run ahead
    bool gen;        // some plane not 16-byte aligned or H*W not a multiple of 4
    unsigned wgs;    // workgroups (a multiple of 8)
    size_t lds_bytes;
};

// Tiling and arguments of a 1x1 convolution without epilogue statistics that one launch covers; false
// if the kernel does not take the layer or the tensors need several launches.  Defined in conv1x1_bf16.hip.
bool conv1x1_bf16_plan(View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g, Epilogue ep,
                       const View *r, View out, C1Launch &L);

namespace {

namespace c1 {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef float f4a_t __attribute__((ext_vector_type(4)));              // 16-byte aligned
typedef float f4u_t __attribute__((ext_vector_type(4), aligned(4)));  // only element aligned
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u2a_t __attribute__((ext_vector_type(2)));  // four bf16, 8-byte aligned

constexpr int kThreads = 256;


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
// IN16 (aligned variant only): `in` holds bf16 already (dense planes, same element strides; no BN
// prologue): the values a conversion on load would produce, so results are the same bits at half the bytes.
template <int MTW, int DEPTH, bool GEN, bool EMIT = false, bool IN16 = false>
__device__ __forceinline__ void conv1x1_bf16_body(const C1Args &p, int bx, int gx, float *red) {
    using F4 = typename std::conditional<GEN, f4u_t, f4a_t>::type;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, kg = lane >> 5;

    // Workgroup ids go round-robin over the 8 dies; give every die a contiguous
    // range of the (pixel tile, channel tile) space so that workgroups sharing
    // input data also share an L2.
    const int per_die = gx >> 3;
    const int logical = (bx & 7) * per_die + (bx >> 3);
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
    static_assert(!(IN16 && GEN), "bf16 input: aligned planes only");
    constexpr int kInBytes = IN16 ? 2 : 4;
    const uint32_t in_off = (uint32_t)(((int64_t)n * p.isn + pix + (int64_t)(kg * 8) * p.isc) * kInBytes);
    const char *const in_base = reinterpret_cast<const char *>(p.in);
    const int64_t isc_b = p.isc * kInBytes;
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

    using Quad = typename std::conditional<IN16, u2a_t, F4>::type;  // four pixels of one channel as loaded
    struct Buf {
        Quad v[8];
        uint4_t a[MTW];
    };
    auto load = [&](Buf &b, int ks) {
#pragma unroll
        for (int k = 0; k < 8; ++k)
            b.v[k] = *reinterpret_cast<const Quad *>(in_base + (int64_t)(ks * 16 + k) * isc_b + in_off);
#pragma unroll
        for (int m = 0; m < MTW; ++m) {
            const bool has = mt0 + m < p.mtiles;
            b.a[m] = *reinterpret_cast<const uint4_t *>(w_base + (has ? m * tile_w : 0) + (int64_t)ks * 1024 + w_off);
        }
    };
    auto compute = [&](Buf &b, int ks) {
        if constexpr (IN16) {
            // dword w of channel k holds pixels 2w, 2w + 1; the operand of pixel j wants the 8 channels in
            // pairs: one byte permute per dword (low halves for even pixels, high halves for odd ones)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
                uint4_t bq;
#pragma unroll
                for (int d = 0; d < 4; ++d) bq[d] = __builtin_amdgcn_perm(b.v[2 * d + 1][j >> 1], b.v[2 * d][j >> 1], sel);
                const bf16x8_t bo = *reinterpret_cast<const bf16x8_t *>(&bq);
#pragma unroll
                for (int m = 0; m < MTW; ++m)
                    acc[m][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8_t *>(&b.a[m]), bo,
                                                                        acc[m][j], 0, 0, 0);
            }
            (void)ks;
            return;
        } else {
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
        // red: [KW - 1][PW * CW][MTW * 64 registers][64 lanes]
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

}  // namespace c1

}  // namespace

}  // namespace rvn
