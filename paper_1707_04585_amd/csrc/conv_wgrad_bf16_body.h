// Kernel body and argument block of the filter gradient with bf16 operands (see
// conv_wgrad_bf16.hip for the design), as a device function so that a launch can
// hold it next to another body.  Device code only.
#pragma once

#include <type_traits>

#include "kernels.h"

namespace rvn {

struct WgArgs {
    const float *x;  // layer input, fp32
    int64_t xsn, xsc;
    const float *scale_shift;  // [2*CI]: a = max(x*scale + shift, 0)
    const float *dh;           // upstream gradient, fp32
    int64_t dsn, dsc;
    float *part;  // [S][tile group][tile][tap][16][64]
    int N, H, W, CI, CO;
    int TH, IMGS, bands, units, upw;  // rows and images per unit, bands per image, units per workgroup
    int Wq, cpr;                      // 4-pixel groups and 8-pixel chunks per image row
    int lrows, a_pitch, a_img, a_plane;  // LDS geometry of a (bf16 elements)
    int d_pitch, d_img, d_plane;         // LDS geometry of dh (bf16 elements)
    int chunks;                          // 8-pixel chunks per unit = IMGS * TH * cpr
    uint32_t m_wq;                       // fast-division multiplier (see fdiv)
    int part_stride;                     // floats of one workgroup column's partial results
};

// What a launch of the filter gradient needs besides its arguments.
struct WgLaunch {
    WgArgs a;
    int KS, MT, CT;
    bool vec;  // every plane 16-byte aligned and the rows whole 4-pixel groups
    dim3 grid;
    size_t lds_bytes;
    WgradReduce red;  // the sum over the workgroups' partial results that has to follow
};

// Tiling and arguments of a filter gradient; false if the kernel does not take the layer.  Defined in
// conv_wgrad_bf16.hip.
bool conv_wgrad_bf16_plan(View x, const float *scale_shift, View dh, int cin, int cout, int ks, Geo g, float *scratch,
                          float *dw, bool accumulate, WgLaunch &L);

namespace {

namespace wg {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef float f4u_t __attribute__((ext_vector_type(4), aligned(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u2w_t __attribute__((ext_vector_type(2)));  // four bf16, 8-byte aligned

constexpr int kThreads = 256;


// e / d for 0 <= e, e * d < 2^32, with m = 2^32 / d + 1 computed on the host
// (m = 0 stands for d = 1).
__device__ __forceinline__ int fdiv(int e, uint32_t m) {  // branch-free: keeps the loads of a batch in one basic block
    const uint32_t one = m == 0u ? 1u : 0u;
    return (int)(__umulhi((uint32_t)e, m) + (uint32_t)e * one);
}

// Two floats to a pair of bf16 (nearest even): one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const float2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<const uint32_t *>(&b);
}

// Four consecutive pixels of a row starting at column col, in two steps so
// that the loads of several items can be in flight together: quad_load issues
// one unconditional 16-byte load (from `safe` where the item is outside the
// tensor; rows have 4 pixels or more, and where fewer than 4 are left the load
// starts `sh` pixels early so that it ends inside the row), quad_fix puts the
// pixels in place, with zeros past the end of the row or for an outside item.
template <bool VEC>
__device__ __forceinline__ f4u_t quad_load(const float *g, bool in, const float *safe, int col, int W, int &sh) {
    sh = VEC || !in ? 0 : col - min(col, W - 4);
    if (VEC) return *reinterpret_cast<const float4_t *>(in ? g : safe);
    return *reinterpret_cast<const f4u_t *>((in ? g : safe) - sh);
}
__device__ __forceinline__ float4 quad_fix(f4u_t x, int sh, bool zero) {
    float4 q;
    q.x = sh == 0 ? x[0] : sh == 1 ? x[1] : sh == 2 ? x[2] : x[3];
    q.y = sh == 0 ? x[1] : sh == 1 ? x[2] : sh == 2 ? x[3] : 0.f;
    q.z = sh == 0 ? x[2] : sh == 1 ? x[3] : 0.f;
    q.w = sh == 0 ? x[3] : 0.f;
    if (zero) q = make_float4(0.f, 0.f, 0.f, 0.f);
    return q;
}

// DH16 (VEC only): `dh` holds bf16 already (dense planes, same element strides): the values the
// conversion while staging would produce, so results are the same bits at half the bytes.
template <int KS, int MT, int CT, bool VEC, bool DH16 = false>
__device__ __forceinline__ void conv_wgrad_bf16_body(const WgArgs &p, int bx, int by, int bz, int gz, uint16_t *smem16) {
    constexpr int KS2 = KS * KS, PAD = KS / 2, LP = KS == 3 ? 8 : 0;  // 3x3: image column 0 sits 8 elements into a tile row
    constexpr int WT = MT * CT, KW = 4 / WT;            // tile owners, pixel shares
    // staging items a thread has in flight: 16-byte fp32 quads, 8-byte bf16 quads (at the 64 -> 64 3x3 layer
    // of the 56x56 bottleneck stack 4 / 4 gave 67.2 us for the shared gradient launch, 8 / 16 65.6, 16 / 16 73.1)
    constexpr int kBatch = 8, kBatch16 = 16;
    static_assert(WT == 1 || WT == 2 || WT == 4, "one tile per wavefront");
    static_assert(VEC || !DH16, "bf16 upstream gradient: aligned planes only");
    uint16_t *a_lds = smem16;
    uint16_t *d_lds = smem16 + CT * 32 * p.a_plane;
    __shared__ float ss_lds[2 * CT * 32];  // scale, shift of this workgroup's input channels

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ko0 = by * (MT * 32), c0 = bz * (CT * 32);
    const int u_begin = bx * p.upw;
    const int u_end = min(p.units, u_begin + p.upw);
    const float *const xp = p.x, *const dp = p.dh;
    const int64_t xsn = p.xsn, dsn = p.dsn;
    const int N = p.N, H = p.H, W = p.W, TH = p.TH, IMGS = p.IMGS, bands = p.bands;

    if (threadIdx.x < 2 * CT * 32) {
        const int half = threadIdx.x / (CT * 32), ch = c0 + threadIdx.x - half * (CT * 32);
        ss_lds[threadIdx.x] = ch < p.CI ? p.scale_shift[half * p.CI + ch] : 0.f;
    }
    // Halo and padding elements of the tiles are never staged: zero both once.
    for (int e = tid; e < (CT * 32 * p.a_plane + MT * 32 * p.d_plane) / 8; e += kThreads)
        reinterpret_cast<uint4_t *>(smem16)[e] = uint4_t{0u, 0u, 0u, 0u};

    // ---- staging.  A channel plane of a unit holds Q = IMGS * rows * Wq items of 4 pixels; lane l of a
    //      wavefront owns items l and l + 64 of every plane (the host keeps Q <= 128), and the wavefront
    //      walks over the channels w, w + 4, ...  What depends on the item -- image, row, column, where it
    //      sits in the LDS plane, how many of its pixels exist -- is worked out once per kernel; per unit a
    //      lane only checks its image and row against the tensor, and per channel everything that changes
    //      is wavefront-uniform (plane base, scale, shift).  (With one flat index per item, decoded by
    //      division for every item of every unit, index arithmetic was three quarters of the kernel's
    //      vector instructions.)
    constexpr int kPass = 2;
    struct Item {
        int off;   // element offset from (first image, first row of the unit, column 0) of a channel plane; pulled back by sh
        int lds;   // element offset in the LDS plane
        int meta;  // image | row << 8 | sh << 20 | valid pixels << 22 | live << 25
    };
    auto make_item = [&](int q, int rows, int row_bias, int pitch, int img_stride_lds, int64_t sn, int lead) {
        Item it{0, 0, 0};
        if (q < IMGS * rows * p.Wq) {
            const int t = fdiv(q, p.m_wq), qx = q - t * p.Wq;
            const int img = t / rows, r = t - img * rows;
            const int col = qx * 4;
            const int sh = VEC ? 0 : col - min(col, W - 4);  // a quad that would run over the row end starts early
            it.off = (int)((int64_t)img * sn) + (r - row_bias) * W + col - sh;
            it.lds = img * img_stride_lds + r * pitch + lead + col;
            it.meta = img | (r << 8) | (sh << 20) | (min(4, W - col) << 22) | (1 << 25);
        }
        return it;
    };
    Item ia[kPass], id[kPass];
#pragma unroll
    for (int ps = 0; ps < kPass; ++ps) {
        ia[ps] = make_item(ps * 64 + lane, p.lrows, PAD, p.a_pitch, p.a_img, xsn, LP);
        id[ps] = make_item(ps * 64 + lane, TH, 0, p.d_pitch, p.d_img, dsn, 0);
    }
    const int nch_a = min(CT * 32, p.CI - c0), nch_d = min(MT * 32, p.CO - ko0);  // channels of the tiles that exist

    // One loaded item of channel cl: BN + ReLU (a only), tail and outside zeros, rounding to bf16, into LDS.
    auto convert_store = [&](f4u_t x, int cl, const Item &it, bool inside, bool bn, uint16_t *lds, int plane) {
        const int meta = it.meta;
        const int sh = (meta >> 20) & 3, nv = (meta >> 22) & 7;
        const float4 q = quad_fix(x, VEC ? 0 : sh, !inside);
        float v0 = q.x, v1 = q.y, v2 = q.z, v3 = q.w;
        if (bn) {
            const float scl = ss_lds[cl], sft = ss_lds[CT * 32 + cl];
            v0 = fmaxf(fmaf(v0, scl, sft), 0.f);
            v1 = fmaxf(fmaf(v1, scl, sft), 0.f);
            v2 = fmaxf(fmaf(v2, scl, sft), 0.f);
            v3 = fmaxf(fmaf(v3, scl, sft), 0.f);
            if (!inside) v0 = v1 = v2 = v3 = 0.f;  // zero outside the image is a(x) = 0, not a(0)
        }
        if (nv < 2) v1 = 0.f;
        if (nv < 3) v2 = 0.f;
        if (nv < 4) v3 = 0.f;
        if ((meta >> 25) & 1) *reinterpret_cast<uint2 *>(lds + cl * plane + it.lds) = make_uint2(pack2(v0, v1), pack2(v2, v3));
    };
    auto item_inside = [&](const Item &it, int n0, int row0, int row_bias) {
        const int meta = it.meta;
        return ((meta >> 25) & 1) && n0 + (meta & 0xff) < N && (unsigned)(row0 + ((meta >> 8) & 0xfff) - row_bias) < (unsigned)H;
    };
    // One tensor of unit (n0, row0), kBatch channels in flight per lane.
    auto stage_planes = [&](const float *base, int64_t sc, int64_t sn, const Item (&items)[kPass], int nch, int quads,
                            int row_bias, int n0, int row0, uint16_t *lds, int plane, bool bn) {
        const float *const ubase = base + (int64_t)n0 * sn + (int64_t)row0 * W;
#pragma unroll
        for (int ps = 0; ps < kPass; ++ps) {
            if (ps * 64 >= quads) break;  // no second item per lane in this plane
            const bool inside = item_inside(items[ps], n0, row0, row_bias);
            const int64_t lo = inside ? (int64_t)items[ps].off : 0;  // (outside: the unit's first element, not used)
            for (int cb = wave; cb < nch; cb += 4 * kBatch) {
                f4u_t x[kBatch];
#pragma unroll
                for (int b = 0; b < kBatch; ++b)
                    x[b] = *reinterpret_cast<const f4u_t *>(ubase + (int64_t)min(cb + 4 * b, nch - 1) * sc + lo);
#pragma unroll
                for (int b = 0; b < kBatch; ++b) {
                    if (cb + 4 * b >= nch) break;
                    convert_store(x[b], cb + 4 * b, items[ps], inside, bn, lds, plane);
                }
            }
        }
    };
    // The same for a tensor that is bf16 already: straight into LDS, zeros for an outside item.
    auto store16 = [&](u2w_t v, int cl, const Item &it, bool inside, uint16_t *lds, int plane) {
        if (!inside) v = u2w_t{0u, 0u};
        if ((it.meta >> 25) & 1) *reinterpret_cast<uint2 *>(lds + cl * plane + it.lds) = make_uint2(v[0], v[1]);
    };
    auto stage_planes16 = [&](const uint16_t *base, int64_t sc, int64_t sn, const Item (&items)[kPass], int nch, int quads,
                              int n0, int row0, uint16_t *lds, int plane) {
        const uint16_t *const ubase = base + (int64_t)n0 * sn + (int64_t)row0 * W;
#pragma unroll
        for (int ps = 0; ps < kPass; ++ps) {
            if (ps * 64 >= quads) break;
            const bool inside = item_inside(items[ps], n0, row0, 0);
            const int64_t lo = inside ? (int64_t)items[ps].off : 0;
            for (int cb = wave; cb < nch; cb += 4 * kBatch16) {
                u2w_t x[kBatch16];
#pragma unroll
                for (int b = 0; b < kBatch16; ++b)
                    x[b] = *reinterpret_cast<const u2w_t *>(ubase + (int64_t)min(cb + 4 * b, nch - 1) * sc + lo);
#pragma unroll
                for (int b = 0; b < kBatch16; ++b) {
                    if (cb + 4 * b >= nch) break;
                    store16(x[b], cb + 4 * b, items[ps], inside, lds, plane);
                }
            }
        }
    };
    const uint16_t *const dp16 = reinterpret_cast<const uint16_t *>(p.dh);
    auto origin = [&](int u, int &n0, int &row0) {
        const int g = u / bands;
        n0 = g * IMGS;
        row0 = (u - g * bands) * TH;
    };
    auto stage = [&](int u) {
        int n0, row0;
        origin(u, n0, row0);
        stage_planes(xp + (int64_t)c0 * p.xsc, p.xsc, xsn, ia, nch_a, IMGS * p.lrows * p.Wq, PAD, n0, row0, a_lds, p.a_plane, true);
        if constexpr (DH16)
            stage_planes16(dp16 + (int64_t)ko0 * p.dsc, p.dsc, dsn, id, nch_d, IMGS * TH * p.Wq, n0, row0, d_lds, p.d_plane);
        else
            stage_planes(dp + (int64_t)ko0 * p.dsc, p.dsc, dsn, id, nch_d, IMGS * TH * p.Wq, 0, n0, row0, d_lds, p.d_plane, false);
    };
    // 1x1 filters (16 accumulator registers): when a plane is one item per lane, every load of a unit is
    // requested at once, one unit ahead, and arrives under the matrix instructions of the unit before.
    constexpr bool kCanPrefetch = KS == 1;
    constexpr int NBA = kCanPrefetch ? CT * 8 : 1, NBD = kCanPrefetch ? MT * 8 : 1;  // channels per wavefront and tile
    const bool prefetch = kCanPrefetch && IMGS * p.lrows * p.Wq <= 64 && IMGS * TH * p.Wq <= 64;
    using DQuad = typename std::conditional<DH16, u2w_t, f4u_t>::type;
    f4u_t pa[NBA];
    DQuad pd[NBD];
    auto request_unit = [&](int u) {
        int n0, row0;
        origin(u, n0, row0);
        const float *const ua = xp + (int64_t)c0 * p.xsc + (int64_t)n0 * xsn + (int64_t)row0 * W +
                                (item_inside(ia[0], n0, row0, PAD) ? (int64_t)ia[0].off : 0);
        const int64_t ud_off = (int64_t)ko0 * p.dsc + (int64_t)n0 * dsn + (int64_t)row0 * W +
                               (item_inside(id[0], n0, row0, 0) ? (int64_t)id[0].off : 0);
#pragma unroll
        for (int b = 0; b < NBA; ++b) pa[b] = *reinterpret_cast<const f4u_t *>(ua + (int64_t)min(wave + 4 * b, nch_a - 1) * p.xsc);
#pragma unroll
        for (int b = 0; b < NBD; ++b) {
            const int64_t o = ud_off + (int64_t)min(wave + 4 * b, nch_d - 1) * p.dsc;
            if constexpr (DH16) pd[b] = *reinterpret_cast<const u2w_t *>(dp16 + o);
            else pd[b] = *reinterpret_cast<const f4u_t *>(dp + o);
        }
    };
    auto commit_unit = [&](int u) {
        int n0, row0;
        origin(u, n0, row0);
        const bool ina = item_inside(ia[0], n0, row0, PAD), ind = item_inside(id[0], n0, row0, 0);
#pragma unroll
        for (int b = 0; b < NBA; ++b)
            if (wave + 4 * b < nch_a) convert_store(pa[b], wave + 4 * b, ia[0], ina, true, a_lds, p.a_plane);
#pragma unroll
        for (int b = 0; b < NBD; ++b)
            if (wave + 4 * b < nch_d) {
                if constexpr (DH16) store16(pd[b], wave + 4 * b, id[0], ind, d_lds, p.d_plane);
                else convert_store(pd[b], wave + 4 * b, id[0], ind, false, d_lds, p.d_plane);
            }
    };

    // ---- this wavefront's tile and share of the steps
    const int tile = wave / KW, kw = wave - tile * KW;
    const int m = tile / CT, ct = tile - m * CT;
    const int l32 = lane & 31, kg = lane >> 5;
    const int a_base = (ct * 32 + l32) * p.a_plane + LP;
    const int d_base = (m * 32 + l32) * p.d_plane;
    const int steps = (p.chunks + 1) >> 1;  // 16-pixel steps per unit (two chunks each)

    float16_t acc[KS2];
#pragma unroll
    for (int t = 0; t < KS2; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    if (prefetch && u_begin < u_end) request_unit(u_begin);
    for (int u = u_begin; u < u_end; ++u) {
        __syncthreads();  // the previous unit has been consumed (first pass: tiles zeroed, ss_lds written)
        if (prefetch) commit_unit(u);
        else stage(u);
        __syncthreads();
        if (prefetch && u + 1 < u_end) request_unit(u + 1);
        // This lane's chunk in step t is q = 2*t + kg -> (image, row, chunk in row).
        int q = 2 * kw + kg, img = 0, row = 0, cr = q;
        for (int t = kw; t < steps; t += KW) {
            while (cr >= p.cpr) {
                cr -= p.cpr;
                ++row;
            }
            while (row >= TH) {
                row -= TH;
                ++img;
            }
            const bool live = q < p.chunks;  // odd chunk count: the last step's second half is empty
            const int doff = live ? d_base + img * p.d_img + row * p.d_pitch + cr * 8 : d_base;
            const int aoff = live ? a_base + img * p.a_img + row * p.a_pitch + cr * 8 : a_base;
            uint4_t dv = *reinterpret_cast<const uint4_t *>(d_lds + doff);
            if (!live) dv = uint4_t{0u, 0u, 0u, 0u};
            const bf16x8_t av = *reinterpret_cast<const bf16x8_t *>(&dv);
#pragma unroll
            for (int rr = 0; rr < KS; ++rr) {
                const uint16_t *rowp = a_lds + aoff + rr * p.a_pitch;
                const uint4_t c = *reinterpret_cast<const uint4_t *>(rowp);
                if (KS == 1) {
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, *reinterpret_cast<const bf16x8_t *>(&c), acc[0], 0, 0, 0);
                } else {
                    const uint32_t prev = *reinterpret_cast<const uint32_t *>(rowp - 2);
                    const uint32_t next = *reinterpret_cast<const uint32_t *>(rowp + 8);
                    // column tap s = 0: pixels -1 .. 6; s = 2: pixels 1 .. 8
                    const uint4_t lft = {__builtin_amdgcn_alignbit(c[0], prev, 16), __builtin_amdgcn_alignbit(c[1], c[0], 16),
                                         __builtin_amdgcn_alignbit(c[2], c[1], 16), __builtin_amdgcn_alignbit(c[3], c[2], 16)};
                    const uint4_t rgt = {__builtin_amdgcn_alignbit(c[1], c[0], 16), __builtin_amdgcn_alignbit(c[2], c[1], 16),
                                         __builtin_amdgcn_alignbit(c[3], c[2], 16), __builtin_amdgcn_alignbit(next, c[3], 16)};
                    acc[rr * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, *reinterpret_cast<const bf16x8_t *>(&lft), acc[rr * 3 + 0], 0, 0, 0);
                    acc[rr * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, *reinterpret_cast<const bf16x8_t *>(&c), acc[rr * 3 + 1], 0, 0, 0);
                    acc[rr * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, *reinterpret_cast<const bf16x8_t *>(&rgt), acc[rr * 3 + 2], 0, 0, 0);
                }
            }
            q += 2 * KW;
            cr += 2 * KW;
        }
    }

    // ---- the workgroup's partial result, in register order [tile][tap][i][lane]
    //      (register i of a lane is dW[m*32 + 8*(i/4) + 4*kg + i%4][ct*32 + l32]);
    //      pixel shares of a tile are summed in a fixed order through LDS, one tap
    //      at a time
    float *out = p.part + (int64_t)bx * p.part_stride +
                 (int64_t)(by * gz + bz) * (WT * KS2 * 1024);
    if (KW == 1) {
#pragma unroll
        for (int t = 0; t < KS2; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) out[((tile * KS2 + t) * 16 + i) * 64 + lane] = acc[t][i];
    } else {
        float *red = reinterpret_cast<float *>(smem16);  // 4 wavefronts x 1024 floats
#pragma unroll
        for (int t = 0; t < KS2; ++t) {
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 16; ++i) red[(wave * 16 + i) * 64 + lane] = acc[t][i];
            __syncthreads();
            for (int idx = tid; idx < WT * 1024; idx += kThreads) {
                const int tl = idx >> 10, rest = idx & 1023;
                float v = red[(tl * KW) * 1024 + rest];
#pragma unroll
                for (int k = 1; k < KW; ++k) v += red[(tl * KW + k) * 1024 + rest];
                out[(tl * KS2 + t) * 1024 + rest] = v;
            }
        }
    }
}

}  // namespace wg

}  // namespace

}  // namespace rvn
