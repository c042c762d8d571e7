// Filter gradient of the units c_k(x) = Conv_kxk(ReLU(BN(x))) (Section 2.2) on
// the CDNA4 matrix cores: the "ordinary backprop" step of Algorithm 1
// (Section 3.2) that produces the derivative with respect to the weights.
//
// GEMM view.  For every filter tap (r, s):
//     dW[ko][c] = sum_pixels dh[ko][pixel] * a[c][pixel + (r - pad, s - pad)]
// i.e. M = output channels, N = input channels, reduction over all N*H*W
// pixels.  One v_mfma_f32_16x16x4_f32 consumes 4 consecutive pixels of one
// image row: its A operand is a 16(ko) x 4(pixel) slice of dh, its B operand a
// 4(pixel) x 16(c) slice of a, shifted by the tap.
//
// Work decomposition.  The pixels are cut into units (TH full rows of IMGS
// images); workgroup s walks over a contiguous range of units and keeps its
// partial sums in registers, so each workgroup writes its share of dW once.
// Inside a workgroup every wavefront owns one 16x16 (ko, c) tile for all k*k
// taps and a 1/KW share of the 4-pixel steps of a unit.  Both operands are
// staged through LDS in NCHW order: dh as is (rounded to bf16 when the
// convolution works on bf16 operands) and a(x) = max(x*scale + shift, 0)
// formed on the way in from the layer input x, with zero halo rows/columns --
// a(x) is never read from HBM.  The global loads of the next unit are issued
// before the matrix instructions of the current one and land in LDS after
// them.  The workgroups' partial results are summed by a second kernel in a
// fixed order (no floating-point atomics: results are bitwise reproducible).
#include "kernels.h"
#include "wgrad_reduce.h"

namespace rvn {

namespace {

typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kItemsA = 8, kItemsD = 5;  // 16-byte LDS items of a / of dh a thread stages per unit (at most)

struct WgradArgs {
    const float *x;  // layer input, fp32
    int64_t xsn, xsc;
    const float *scale_shift;  // [2*CI]: a = max(x*scale + shift, 0)
    const float *dh;           // upstream gradient, fp32
    int64_t dsn, dsc;
    float *part;  // [S][CO][CI][KS*KS]
    int N, H, W, CI, CO;
    int round_bf16;
    int TH, IMGS, bands, units, upw;  // rows and images per unit, bands per image, units per workgroup
    int Wq;                           // 4-pixel groups per image row
    int lrows, a_pitch, a_img, a_plane;  // LDS geometry of a (floats)
    int d_pitch, d_img, d_plane;         // LDS geometry of dh (floats)
    int a_items, d_items;                // 16-byte items per unit
    int steps_per_img, steps;            // 4-pixel steps per image / per unit
    uint32_t m_aq, m_lrows, m_imgs, m_wq, m_th;  // fast-division multipliers (see fdiv)
    int part_stride;                     // floats of one workgroup column's partial results
};

// e / d for 0 <= e, e * d < 2^32, with m = 2^32 / d + 1 computed on the host
// (m = 0 stands for d = 1).
__device__ __forceinline__ int fdiv(int e, uint32_t m) { return m ? (int)__umulhi((uint32_t)e, m) : e; }

__device__ __forceinline__ float bf16_round_dev(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f;
    u += 0x7fffu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xffff0000u);
}

// One 16-byte item of an LDS tile: where it goes, where it comes from, and the
// unit-independent part of its validity.
struct Item {
    int dst;    // LDS offset in floats, -1: this thread has no such item
    int src;    // offset inside an image: channel * channel stride + column
    int where;  // image in unit | (row offset + 1) << 8 | loaded << 20 | channel and column valid << 21 | local channel << 22
};

// Four consecutive floats of a row starting at column `col`.  The fast path
// (16-byte aligned rows, W a multiple of 4) always issues the load -- from a
// harmless address when the item lies outside the tensor -- so that no branch,
// and with it no wait, separates the loads of a unit; the caller zeroes such
// items when it writes them to LDS.
template <bool VEC>
__device__ __forceinline__ float4 load_quad(const float *g, bool in, const float *safe, int col, int W) {
    if (VEC) return *reinterpret_cast<const float4 *>(in ? g : safe);
    float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
    if (in) {
        q.x = g[0];
        if (col + 1 < W) q.y = g[1];
        if (col + 2 < W) q.z = g[2];
        if (col + 3 < W) q.w = g[3];
    }
    return q;
}

template <int KS, int MT, int CT, bool VEC>
__global__ __launch_bounds__(kThreads) void conv_wgrad_mfma_k(const WgradArgs p) {
    constexpr int KS2 = KS * KS, PAD = KS / 2, LP = KS == 3 ? 4 : 0;
    constexpr int WT = MT * CT, KW = 4 / WT;  // tile owners, pixel shares
    static_assert(WT == 1 || WT == 2 || WT == 4, "one tile per wavefront");
    extern __shared__ __align__(16) float smem[];
    float *a_lds = smem;
    float *d_lds = smem + CT * 16 * p.a_plane;
    __shared__ float ss_lds[2 * CT * 16];  // scale, shift of this workgroup's input channels

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ko0 = blockIdx.y * (MT * 16), c0 = blockIdx.z * (CT * 16);
    const int u_begin = blockIdx.x * p.upw;
    const int u_end = min(p.units, u_begin + p.upw);
    const float *const xp = p.x, *const dp = p.dh;
    const int64_t xsn = p.xsn, dsn = p.dsn;
    const int N = p.N, H = p.H, W = p.W, TH = p.TH, IMGS = p.IMGS, bands = p.bands;
    const bool round_bf16 = p.round_bf16 != 0;

    if (threadIdx.x < 2 * CT * 16) {
        const int half = threadIdx.x / (CT * 16), ch = c0 + threadIdx.x - half * (CT * 16);
        ss_lds[threadIdx.x] = ch < p.CI ? p.scale_shift[half * p.CI + ch] : 0.f;
    }
    // ---- what this thread stages for every unit (independent of the unit)
    Item ia[kItemsA], id[kItemsD];
    {
        const int aq = p.a_pitch >> 2;
#pragma unroll
        for (int i = 0; i < kItemsA; ++i) {
            const int e = tid + i * kThreads;
            ia[i] = Item{-1, 0, 0};
            if (e < p.a_items) {
                const int t = fdiv(e, p.m_aq), qx = e - t * aq;
                const int t2 = fdiv(t, p.m_lrows), lr = t - t2 * p.lrows;
                const int cl = fdiv(t2, p.m_imgs), img = t2 - cl * IMGS;
                const int col = qx * 4 - LP, ch = c0 + cl;
                const bool ok = ch < p.CI && col >= 0 && col < W;
                ia[i].dst = cl * p.a_plane + img * p.a_img + lr * p.a_pitch + qx * 4;
                ia[i].src = ch * (int)p.xsc + col;
                ia[i].where = img | ((lr - PAD + 1) << 8) | (ok ? 1 << 21 : 0) | (cl << 22);
            }
        }
#pragma unroll
        for (int i = 0; i < kItemsD; ++i) {
            const int e = tid + i * kThreads;
            id[i] = Item{-1, 0, 0};
            if (e < p.d_items) {
                const int t = fdiv(e, p.m_wq), qx = e - t * p.Wq;
                const int t2 = fdiv(t, p.m_th), r = t - t2 * TH;
                const int ml = fdiv(t2, p.m_imgs), img = t2 - ml * IMGS;
                const int col = qx * 4, ko = ko0 + ml;
                const bool ok = ko < p.CO && col < W;
                id[i].dst = CT * 16 * p.a_plane + ml * p.d_plane + img * p.d_img + r * p.d_pitch + qx * 4;
                id[i].src = ko * (int)p.dsc + col;
                id[i].where = img | ((r + 1) << 8) | (ok ? 1 << 21 : 0);
            }
        }
    }

    float4 qa[kItemsA], qd[kItemsD];
    // Issue the global loads of unit u; items outside the tensor stay zero.
    auto prefetch = [&](int u) {
        const int g = u / bands;
        const int n0 = g * IMGS, row0 = (u - g * bands) * TH;
#pragma unroll
        for (int i = 0; i < kItemsA; ++i) {
            const int n = n0 + (ia[i].where & 0xff), row = row0 + ((ia[i].where >> 8) & 0xfff) - 1;
            const bool in = (ia[i].where & (1 << 21)) && n < N && row >= 0 && row < H;
            qa[i] = load_quad<VEC>(xp + (int64_t)n * xsn + ia[i].src + row * W, in, xp, VEC ? 0 : ia[i].src % (int)p.xsc, W);
            ia[i].where = in ? ia[i].where | (1 << 20) : ia[i].where & ~(1 << 20);  // bit 20: loaded
        }
#pragma unroll
        for (int i = 0; i < kItemsD; ++i) {
            const int n = n0 + (id[i].where & 0xff), row = row0 + ((id[i].where >> 8) & 0xfff) - 1;
            const bool in = (id[i].where & (1 << 21)) && n < N && row < H;
            qd[i] = load_quad<VEC>(dp + (int64_t)n * dsn + id[i].src + row * W, in, dp, VEC ? 0 : id[i].src % (int)p.dsc, W);
            id[i].where = in ? id[i].where | (1 << 20) : id[i].where & ~(1 << 20);
        }
    };
    // Write the loaded unit to LDS: a = max(x*scale + shift, 0) (zero outside the
    // image), dh as is; both rounded to bf16 if the convolution asks for it.
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < kItemsA; ++i) {
            if (ia[i].dst < 0) continue;
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (ia[i].where & (1 << 20)) {  // loaded from inside the tensor
                v[0] = qa[i].x; v[1] = qa[i].y; v[2] = qa[i].z; v[3] = qa[i].w;
                const int cl = (ia[i].where >> 22) & 31;
                const float sc = ss_lds[cl], sh = ss_lds[CT * 16 + cl];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    v[j] = fmaxf(fmaf(v[j], sc, sh), 0.f);
                    if (round_bf16) v[j] = bf16_round_dev(v[j]);
                }
                if (!VEC) {  // a(x) past the right image border is zero, not max(shift, 0)
                    const int col = ia[i].src % (int)p.xsc;
#pragma unroll
                    for (int j = 1; j < 4; ++j)
                        if (col + j >= W) v[j] = 0.f;
                }
            }
            *reinterpret_cast<float4 *>(smem + ia[i].dst) = make_float4(v[0], v[1], v[2], v[3]);
        }
#pragma unroll
        for (int i = 0; i < kItemsD; ++i) {
            if (id[i].dst < 0) continue;
            const bool in = id[i].where & (1 << 20);
            float v[4] = {in ? qd[i].x : 0.f, in ? qd[i].y : 0.f, in ? qd[i].z : 0.f, in ? qd[i].w : 0.f};
            if (round_bf16) {
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = bf16_round_dev(v[j]);
            }
            *reinterpret_cast<float4 *>(smem + id[i].dst) = make_float4(v[0], v[1], v[2], v[3]);
        }
    };

    // ---- this wavefront's tile and share of the steps
    const int tile = wave / KW, kw = wave - tile * KW;
    const int m = tile / CT, ct = tile - m * CT;
    const int l16 = lane & 15, kq = lane >> 4;
    const int a_base = (ct * 16 + l16) * p.a_plane + (LP - PAD) + kq;
    const int d_base = (m * 16 + l16) * p.d_plane + kq;

    float4_t acc[KS2];
#pragma unroll
    for (int t = 0; t < KS2; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};

    if (u_begin < u_end) prefetch(u_begin);
    for (int u = u_begin; u < u_end; ++u) {
        __syncthreads();  // the previous unit has been consumed
        commit();
        __syncthreads();
        if (u + 1 < u_end) prefetch(u + 1);
        // Operands of step t+KW are read from LDS before the matrix
        // instructions of step t are issued.
        int img = 0, row = 0, cq = kw;
        auto offsets = [&](int &ao, int &dof) {
            while (cq >= p.Wq) {
                cq -= p.Wq;
                ++row;
            }
            while (row >= TH) {
                row -= TH;
                ++img;
            }
            ao = a_base + img * p.a_img + row * p.a_pitch + cq * 4;
            dof = d_base + img * p.d_img + row * p.d_pitch + cq * 4;
            cq += KW;
        };
        float av, bv[KS2];
        auto read_operands = [&](int ao, int dof) {
            av = d_lds[dof];
#pragma unroll
            for (int rr = 0; rr < KS; ++rr)
#pragma unroll
                for (int ss = 0; ss < KS; ++ss) bv[rr * KS + ss] = a_lds[ao + rr * p.a_pitch + ss];
        };
        if (kw < p.steps) {
            int ao, dof;
            offsets(ao, dof);
            read_operands(ao, dof);
        }
        for (int t = kw; t < p.steps; t += KW) {
            const float av0 = av;
            float bv0[KS2];
#pragma unroll
            for (int i = 0; i < KS2; ++i) bv0[i] = bv[i];
            if (t + KW < p.steps) {
                int ao, dof;
                offsets(ao, dof);
                read_operands(ao, dof);
            }
#pragma unroll
            for (int i = 0; i < KS2; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av0, bv0[i], acc[i], 0, 0, 0);
        }
    }

    // ---- sum the KW pixel shares of every tile in a fixed order and write the
    //      workgroup's partial result: lane holds dW[m*16 + 4*kq + j][ct*16 + l16]
    __syncthreads();
    float *red = smem;
#pragma unroll
    for (int t = 0; t < KS2; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) red[((wave * KS2 + t) * 4 + j) * 64 + lane] = acc[t][j];
    __syncthreads();
    // Partial results keep the register order [tile][tap][j][lane]; the reduce
    // kernel maps it to [ko][c][tap].
    float *out = p.part + (int64_t)blockIdx.x * p.part_stride +
                 (int64_t)(blockIdx.y * gridDim.z + blockIdx.z) * (WT * KS2 * 256);
    for (int idx = tid; idx < WT * KS2 * 256; idx += kThreads) {
        const int tl = idx / (KS2 * 256), rest = idx - tl * (KS2 * 256);
        float v = red[(tl * KW) * KS2 * 256 + rest];
#pragma unroll
        for (int k = 1; k < KW; ++k) v += red[(tl * KW + k) * KS2 * 256 + rest];
        out[idx] = v;
    }
}

__global__ __launch_bounds__(kThreads) void wgrad_reduce_k(const WgradReduce r) {
    __shared__ float lds[kThreads];
    wgrad_reduce_body(r, blockIdx.x, lds);
}

struct WgradPlan {
    int MT, CT, TH, IMGS, bands, units, S, upw, Wq, lrows;
    int a_pitch, a_img, a_plane, d_pitch, d_img, d_plane, a_items, d_items;
    size_t lds_bytes;
    int tiles_ko, tiles_c, part_stride;
    bool ok;
};

uint32_t fdiv_magic(int d) { return d == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)d + 1ull); }


int bank_pad(int plane) {  // smallest value >= plane that is 4 modulo 64
    return plane + ((4 - plane % 64) + 64) % 64;
}

WgradPlan plan_wgrad(int cin, int cout, int ks, const Geo &g) {
    WgradPlan w{};
    w.MT = cout <= 16 ? 1 : 2;
    w.CT = cin <= 16 ? 1 : 2;
    const int lp = ks == 3 ? 4 : 0;
    w.Wq = (g.w + 3) / 4;
    w.a_pitch = lp + 4 * w.Wq + (ks == 3 ? 4 : 0);
    w.d_pitch = 4 * w.Wq;
    w.tiles_ko = (cout + w.MT * 16 - 1) / (w.MT * 16);
    w.tiles_c = (cin + w.CT * 16 - 1) / (w.CT * 16);
    const size_t red_bytes = (size_t)4 * ks * ks * 256 * 4;
    // Largest unit that fits: whole images if possible, else the tallest band.
    auto fits = [&](int th, int imgs) {
        const int lrows = th + ks - 1;
        const int a_img = lrows * w.a_pitch, d_img = th * w.d_pitch;
        const int a_plane = bank_pad(imgs * a_img), d_plane = bank_pad(imgs * d_img);
        const int a_items = w.CT * 16 * imgs * lrows * (w.a_pitch / 4);
        const int d_items = w.MT * 16 * imgs * th * w.Wq;
        const size_t bytes = ((size_t)w.CT * 16 * a_plane + (size_t)w.MT * 16 * d_plane) * 4;
        if (a_items > kItemsA * kThreads || d_items > kItemsD * kThreads || bytes > 64 * 1024 || imgs > 255 || lrows > 4000) return false;
        w.TH = th; w.IMGS = imgs; w.lrows = lrows;
        w.a_img = a_img; w.d_img = d_img; w.a_plane = a_plane; w.d_plane = d_plane;
        w.a_items = a_items; w.d_items = d_items;
        w.lds_bytes = bytes > red_bytes ? bytes : red_bytes;
        return true;
    };
    w.ok = false;
    for (int imgs = g.n < 8 ? g.n : 8; imgs >= 1 && !w.ok; --imgs) w.ok = fits(g.h, imgs);
    for (int th = g.h - 1; th >= 1 && !w.ok; --th) w.ok = fits(th, 1);
    if (!w.ok) return w;
    if (w.IMGS == 1) {  // equal bands: no taller than what fits, as few as that allows
        const int bands = (g.h + w.TH - 1) / w.TH;
        fits((g.h + bands - 1) / bands, 1);
    }
    w.bands = (g.h + w.TH - 1) / w.TH;
    w.units = ((g.n + w.IMGS - 1) / w.IMGS) * w.bands;
    const int groups = w.tiles_ko * w.tiles_c;
    w.part_stride = groups * w.MT * w.CT * ks * ks * 256;
    int s = 256 / groups;  // one workgroup per compute unit
    if (s < 1) s = 1;
    if (s > w.units) s = w.units;
    w.upw = (w.units + s - 1) / s;
    w.S = (w.units + w.upw - 1) / w.upw;
    return w;
}

}  // namespace

size_t wgrad_scratch_floats(int cin, int cout, int ks, const Geo &g) {
    const WgradPlan w = plan_wgrad(cin, cout, ks, g);
    const size_t a = w.ok ? (size_t)w.S * w.part_stride : 0, b = wgrad_bf16_scratch_floats(cin, cout, ks, g);
    return a > b ? a : b;
}

void conv_wgrad(Ctx &cx, View x, const float *scale_shift, rvn_dtype dt, View dh, int cin, int cout,
                int ks, Geo g, float *scratch, float *dw, bool accumulate, WgradReduce *defer) {
    if (defer) defer->blocks = 0;
    const double P = (double)g.pixels();
    const double flops = 2.0 * P * cin * cout * ks * ks;
    cx.cost.conv_wgrad_calls += 1;
    cx.cost.conv_flops += flops;
    if (dt == RVN_BF16 &&
        conv_wgrad_bf16(cx, x, scale_shift, dh, cin, cout, ks, g, scratch, dw, accumulate,
                        P * cin * 4.0 + P * cout * 4.0, flops, defer))
        return;
    const WgradPlan w = plan_wgrad(cin, cout, ks, g);
    if (cx.launch(K_CONV_WGRAD, P * cin * 4.0 + P * cout * 4.0, flops)) {
        if (!w.ok) {  // image rows too wide for LDS
            cx.fail(hipErrorInvalidConfiguration);
            return;
        }
        WgradArgs a{};
        a.x = x.p; a.xsn = x.sn; a.xsc = x.sc;
        a.scale_shift = scale_shift;
        a.dh = dh.p; a.dsn = dh.sn; a.dsc = dh.sc;
        a.part = scratch;
        a.N = g.n; a.H = g.h; a.W = g.w; a.CI = cin; a.CO = cout;
        a.round_bf16 = dt == RVN_BF16 ? 1 : 0;
        a.TH = w.TH; a.IMGS = w.IMGS; a.bands = w.bands; a.units = w.units; a.upw = w.upw;
        a.Wq = w.Wq; a.lrows = w.lrows;
        a.a_pitch = w.a_pitch; a.a_img = w.a_img; a.a_plane = w.a_plane;
        a.d_pitch = w.d_pitch; a.d_img = w.d_img; a.d_plane = w.d_plane;
        a.a_items = w.a_items; a.d_items = w.d_items;
        a.steps_per_img = w.TH * w.Wq;
        a.steps = w.IMGS * w.TH * w.Wq;
        a.m_aq = fdiv_magic(w.a_pitch / 4); a.m_lrows = fdiv_magic(w.lrows); a.m_imgs = fdiv_magic(w.IMGS);
        a.m_wq = fdiv_magic(w.Wq); a.m_th = fdiv_magic(w.TH);
        a.part_stride = w.part_stride;
        dim3 grid((unsigned)w.S, (unsigned)w.tiles_ko, (unsigned)w.tiles_c);
        const bool vec = (g.w & 3) == 0 && (x.sn & 3) == 0 && (x.sc & 3) == 0 && (dh.sn & 3) == 0 &&
                         (dh.sc & 3) == 0 && (reinterpret_cast<uintptr_t>(x.p) & 15) == 0 &&
                         (reinterpret_cast<uintptr_t>(dh.p) & 15) == 0;
#define RVN_CASE(KS_, MT_, CT_)                                                                    \
    if (ks == KS_ && w.MT == MT_ && w.CT == CT_) {                                                 \
        if (vec) cx.run(conv_wgrad_mfma_k<KS_, MT_, CT_, true>, grid, dim3(kThreads), w.lds_bytes, a);   \
        else cx.run(conv_wgrad_mfma_k<KS_, MT_, CT_, false>, grid, dim3(kThreads), w.lds_bytes, a);      \
    }
        RVN_CASE(3, 1, 1) RVN_CASE(3, 1, 2) RVN_CASE(3, 2, 1) RVN_CASE(3, 2, 2)
        RVN_CASE(1, 1, 1) RVN_CASE(1, 1, 2) RVN_CASE(1, 2, 1) RVN_CASE(1, 2, 2)
#undef RVN_CASE
    }
    WgradReduce red{};
    red.part = scratch; red.dw = dw;
    red.part_stride = w.part_stride; red.S = w.S; red.KS2 = ks * ks; red.MT = w.MT; red.CT = w.CT;
    red.tiles_c = w.tiles_c; red.CO = cout; red.CI = cin; red.accumulate = accumulate ? 1 : 0;
    red.tile = 16; red.blocks = (w.part_stride + 31) / 32;
    if (defer) *defer = red;
    else wgrad_reduce(cx, red);
}

void wgrad_reduce(Ctx &cx, const WgradReduce &r) {
    if (r.blocks <= 0) return;
    if (cx.launch(K_WGRAD_REDUCE, 0.0)) cx.run(wgrad_reduce_k, dim3((unsigned)r.blocks), dim3(kThreads), 0, r);
}

}  // namespace rvn
