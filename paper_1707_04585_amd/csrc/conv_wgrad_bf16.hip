// Filter gradient with bf16 operands on the CDNA4 matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation): the "ordinary backprop" step of
// Algorithm 1 (Section 3.2) that produces the derivative with respect to the
// weights, when the block descriptor asks for bf16 convolution operands.
//
// GEMM view.  For every filter tap (r, s):
//     dW[ko][c] = sum_pixels dh[ko][pixel] * a[c][pixel + (r - pad, s - pad)]
// M = output channels, N = input channels, reduction over all N*H*W pixels.
// One matrix instruction consumes 16 pixels: each lane feeds 8 consecutive
// pixels of one image row for its channel, so both operands live in LDS as
// bf16 NCHW planes (pixel innermost) cut into chunks of 8 pixels, and a chunk
// is one aligned 16-byte read.  A tap that moves one column left or right would
// need a misaligned chunk; it is assembled in registers instead from the
// aligned chunk and one dword of its neighbour (four funnel shifts), so the
// activation tile is stored once, with 8 zero elements before and after every
// row for the halo columns.
//
// Work decomposition as in the fp32 kernel: units of TH full rows of IMGS
// images; workgroup s walks over a contiguous range of units with its partial
// sums in registers; every wavefront owns one 32x32 (ko, c) tile for all k*k
// taps and a 1/KW share of the 16-pixel steps; a(x) = max(x*scale + shift, 0) is
// formed (and rounded to bf16) on the way into LDS.  Partial results are summed
// in a fixed order by wgrad_reduce_body, in a launch of its own or carried by
// another kernel.
#include "kernels.h"

namespace rvn {

namespace {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef float f4u_t __attribute__((ext_vector_type(4), aligned(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

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
    int a_items, d_items;                // 4-pixel items per unit
    int chunks;                          // 8-pixel chunks per unit = IMGS * TH * cpr
    uint32_t m_wq, m_lrows, m_imgs, m_th;  // fast-division multipliers (see fdiv)
    int part_stride;                     // floats of one workgroup column's partial results
};

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

template <int KS, int MT, int CT, bool VEC>
__global__ __launch_bounds__(kThreads, 2) void conv_wgrad_bf16_k(const WgArgs p) {
    constexpr int KS2 = KS * KS, PAD = KS / 2, LP = KS == 3 ? 8 : 0;  // 3x3: image column 0 sits 8 elements into a tile row
    constexpr int WT = MT * CT, KW = 4 / WT;            // tile owners, pixel shares
    constexpr int kBatch = KS == 3 ? 4 : 8;             // staging items a thread has in flight
    static_assert(WT == 1 || WT == 2 || WT == 4, "one tile per wavefront");
    extern __shared__ __align__(16) uint16_t smem16[];
    uint16_t *a_lds = smem16;
    uint16_t *d_lds = smem16 + CT * 32 * p.a_plane;
    __shared__ float ss_lds[2 * CT * 32];  // scale, shift of this workgroup's input channels

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ko0 = blockIdx.y * (MT * 32), c0 = blockIdx.z * (CT * 32);
    const int u_begin = blockIdx.x * p.upw;
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

    // Stage unit u: a = max(x*scale + shift, 0) (zero outside the image) and dh,
    // both as bf16, 4 pixels per item.  Several workgroups share a compute unit,
    // so one's loads overlap another's matrix instructions.
    // Items are handled kBatch at a time: all loads of a batch are issued (from a
    // safe address where the item is outside the tensor) before any is converted,
    // so a unit costs a few memory round trips instead of one per item.
    auto stage = [&](int u) {
        const int g = u / bands;
        const int n0 = g * IMGS, row0 = (u - g * bands) * TH;
        for (int e0 = tid; e0 < p.a_items; e0 += kThreads * kBatch) {
            f4u_t x[kBatch];
            int where[kBatch];  // LDS offset (elements) | sh << 20 | outside << 30; negative: no item
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const int e = e0 + b * kThreads;
                const int t = fdiv(e, p.m_wq), qx = e - t * p.Wq;
                const int t2 = fdiv(t, p.m_lrows), lr = t - t2 * p.lrows;
                const int cl = fdiv(t2, p.m_imgs), img = t2 - cl * IMGS;
                const int col = qx * 4, ch = c0 + cl, n = n0 + img, row = row0 - PAD + lr;
                const bool in = e < p.a_items && ch < p.CI && n < N && row >= 0 && row < H;
                int sh;
                x[b] = quad_load<VEC>(xp + (int64_t)n * xsn + (int64_t)ch * p.xsc + row * W + col, in, xp, col, W, sh);
                where[b] = e < p.a_items ? (cl * p.a_plane + img * p.a_img + lr * p.a_pitch + LP + col) | (sh << 20) | (in ? 0 : 1 << 30) : -1;
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const int off = where[b] & 0xfffff;
                const float4 q = quad_fix(x[b], VEC ? 0 : (where[b] >> 20) & 3, false);
                const bool zero = (where[b] >> 30) & 1;
                const int e = e0 + b * kThreads;
                const int t = fdiv(e, p.m_wq), col = (e - t * p.Wq) * 4;
                const int cl = min(fdiv(fdiv(t, p.m_lrows), p.m_imgs), CT * 32 - 1);
                const float sc = ss_lds[cl], sh = ss_lds[CT * 32 + cl];
                const float v0 = zero ? 0.f : fmaxf(fmaf(q.x, sc, sh), 0.f);
                const float v1 = zero || col + 1 >= W ? 0.f : fmaxf(fmaf(q.y, sc, sh), 0.f);
                const float v2 = zero || col + 2 >= W ? 0.f : fmaxf(fmaf(q.z, sc, sh), 0.f);
                const float v3 = zero || col + 3 >= W ? 0.f : fmaxf(fmaf(q.w, sc, sh), 0.f);
                if (where[b] >= 0) *reinterpret_cast<uint2 *>(a_lds + off) = make_uint2(pack2(v0, v1), pack2(v2, v3));
            }
        }
        for (int e0 = tid; e0 < p.d_items; e0 += kThreads * kBatch) {
            f4u_t x[kBatch];
            int where[kBatch];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const int e = e0 + b * kThreads;
                const int t = fdiv(e, p.m_wq), qx = e - t * p.Wq;
                const int t2 = fdiv(t, p.m_th), r = t - t2 * TH;
                const int ml = fdiv(t2, p.m_imgs), img = t2 - ml * IMGS;
                const int col = qx * 4, ko = ko0 + ml, n = n0 + img, row = row0 + r;
                const bool in = e < p.d_items && ko < p.CO && n < N && row < H;
                int sh;
                x[b] = quad_load<VEC>(dp + (int64_t)n * dsn + (int64_t)ko * p.dsc + row * W + col, in, dp, col, W, sh);
                where[b] = e < p.d_items ? (ml * p.d_plane + img * p.d_img + r * p.d_pitch + col) | (sh << 20) | (in ? 0 : 1 << 30) : -1;
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const float4 q = quad_fix(x[b], VEC ? 0 : (where[b] >> 20) & 3, (where[b] >> 30) & 1);
                const uint2 v = make_uint2(pack2(q.x, q.y), pack2(q.z, q.w));
                if (where[b] >= 0) *reinterpret_cast<uint2 *>(d_lds + (where[b] & 0xfffff)) = v;
            }
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

    for (int u = u_begin; u < u_end; ++u) {
        __syncthreads();  // the previous unit has been consumed (first pass: tiles zeroed, ss_lds written)
        stage(u);
        __syncthreads();
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
    float *out = p.part + (int64_t)blockIdx.x * p.part_stride +
                 (int64_t)(blockIdx.y * gridDim.z + blockIdx.z) * (WT * KS2 * 1024);
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

struct WgPlan {
    int MT, CT, TH, IMGS, bands, units, S, upw, Wq, cpr, lrows;
    int a_pitch, a_img, a_plane, d_pitch, d_img, d_plane, a_items, d_items;
    size_t lds_bytes;
    int tiles_ko, tiles_c, part_stride;
    bool ok;
};

uint32_t fdiv_magic(int d) { return d == 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)d + 1ull); }

// Smallest value >= plane that is 8 modulo 16 (elements): planes an odd multiple
// of 16 bytes apart put the 16-byte reads of 8 neighbouring lanes on distinct banks.
int bank_pad(int plane) { return plane + ((8 - plane % 16) + 16) % 16; }

WgPlan plan_wg(int cin, int cout, int ks, const Geo &g) {
    WgPlan w{};
    w.ok = false;
    if (g.w < 4) return w;  // staging loads 4 pixels of a row at a time
    // A 16 x 16 filter fills a quarter of a 32 x 32 result tile; the fp32-instruction
    // kernel (16 x 16 tiles, operands rounded to bf16 on the way in) is faster there.
    if (cin <= 16 && cout <= 16) return w;
    w.MT = cout <= 32 ? 1 : 2;
    w.CT = cin <= 32 ? 1 : 2;
    w.Wq = (g.w + 3) / 4;
    w.cpr = (g.w + 7) / 8;
    w.a_pitch = ks == 3 ? 8 + w.cpr * 8 + 8 : w.cpr * 8;  // 3x3: 8 zero elements before and after every row
    w.d_pitch = w.cpr * 8;
    w.tiles_ko = (cout + w.MT * 32 - 1) / (w.MT * 32);
    w.tiles_c = (cin + w.CT * 32 - 1) / (w.CT * 32);
    const size_t red_bytes = (size_t)4 * 1024 * 4;
    // Largest unit that fits: whole images if possible, else the tallest band.
    auto fits = [&](int th, int imgs) {
        const int lrows = th + ks - 1;
        const int a_img = lrows * w.a_pitch, d_img = th * w.d_pitch;
        const int a_plane = bank_pad(imgs * a_img), d_plane = bank_pad(imgs * d_img);
        const int a_items = w.CT * 32 * imgs * lrows * w.Wq;
        const int d_items = w.MT * 32 * imgs * th * w.Wq;
        const size_t bytes = ((size_t)w.CT * 32 * a_plane + (size_t)w.MT * 32 * d_plane) * 2;
        if (bytes > 64 * 1024 || imgs > 255 || lrows > 4000) return false;
        w.TH = th; w.IMGS = imgs; w.lrows = lrows;
        w.a_img = a_img; w.d_img = d_img; w.a_plane = a_plane; w.d_plane = d_plane;
        w.a_items = a_items; w.d_items = d_items;
        w.lds_bytes = bytes > red_bytes ? bytes : red_bytes;
        return true;
    };
    w.ok = false;
    for (int imgs = g.n < 16 ? g.n : 16; imgs >= 1 && !w.ok; --imgs) w.ok = fits(g.h, imgs);
    for (int th = g.h - 1; th >= 1 && !w.ok; --th) w.ok = fits(th, 1);
    if (!w.ok) return w;
    if (w.IMGS == 1) {  // equal bands: no taller than what fits, as few as that allows
        const int bands = (g.h + w.TH - 1) / w.TH;
        fits((g.h + bands - 1) / bands, 1);
    }
    w.bands = (g.h + w.TH - 1) / w.TH;
    w.units = ((g.n + w.IMGS - 1) / w.IMGS) * w.bands;
    const int groups = w.tiles_ko * w.tiles_c;
    w.part_stride = groups * w.MT * w.CT * ks * ks * 1024;
    // Two workgroups per compute unit.  Fewer slices or 32 x 32 tiles would write fewer partial results, but
    // measured slower on every workload (the launch is bound by staging and the multiply chain, not by those bytes).
    int s = 512 / groups;
    if (s < 1) s = 1;
    if (s > w.units) s = w.units;
    w.upw = (w.units + s - 1) / s;
    w.S = (w.units + w.upw - 1) / w.upw;
    return w;
}

}  // namespace

size_t wgrad_bf16_scratch_floats(int cin, int cout, int ks, const Geo &g) {
    const WgPlan w = plan_wg(cin, cout, ks, g);
    return w.ok ? (size_t)w.S * w.part_stride : 0;
}

bool conv_wgrad_bf16(Ctx &cx, View x, const float *scale_shift, View dh, int cin, int cout, int ks, Geo g,
                     float *scratch, float *dw, bool accumulate, double bytes, double flops, WgradReduce *defer) {
    const WgPlan w = plan_wg(cin, cout, ks, g);
    if (!w.ok) return false;
    WgArgs a{};
    a.x = x.p; a.xsn = x.sn; a.xsc = x.sc;
    a.scale_shift = scale_shift;
    a.dh = dh.p; a.dsn = dh.sn; a.dsc = dh.sc;
    a.part = scratch;
    a.N = g.n; a.H = g.h; a.W = g.w; a.CI = cin; a.CO = cout;
    a.TH = w.TH; a.IMGS = w.IMGS; a.bands = w.bands; a.units = w.units; a.upw = w.upw;
    a.Wq = w.Wq; a.cpr = w.cpr; a.lrows = w.lrows;
    a.a_pitch = w.a_pitch; a.a_img = w.a_img; a.a_plane = w.a_plane;
    a.d_pitch = w.d_pitch; a.d_img = w.d_img; a.d_plane = w.d_plane;
    a.a_items = w.a_items; a.d_items = w.d_items;
    a.chunks = w.IMGS * w.TH * w.cpr;
    a.m_wq = fdiv_magic(w.Wq); a.m_lrows = fdiv_magic(w.lrows); a.m_imgs = fdiv_magic(w.IMGS); a.m_th = fdiv_magic(w.TH);
    a.part_stride = w.part_stride;
    const dim3 grid((unsigned)w.S, (unsigned)w.tiles_ko, (unsigned)w.tiles_c);
    const bool vec = (g.w & 3) == 0 && (x.sn & 3) == 0 && (x.sc & 3) == 0 && (dh.sn & 3) == 0 && (dh.sc & 3) == 0 &&
                     (reinterpret_cast<uintptr_t>(x.p) & 15) == 0 && (reinterpret_cast<uintptr_t>(dh.p) & 15) == 0;
    if (cx.launch(K_CONV_WGRAD, bytes, flops)) {
#define RVN_CASE(KS_, MT_, CT_)                                                                       \
    if (ks == KS_ && w.MT == MT_ && w.CT == CT_) {                                                    \
        if (vec) cx.run(conv_wgrad_bf16_k<KS_, MT_, CT_, true>, grid, dim3(kThreads), w.lds_bytes, a);  \
        else cx.run(conv_wgrad_bf16_k<KS_, MT_, CT_, false>, grid, dim3(kThreads), w.lds_bytes, a);     \
    }
        RVN_CASE(3, 1, 1) RVN_CASE(3, 1, 2) RVN_CASE(3, 2, 1) RVN_CASE(3, 2, 2)
        RVN_CASE(1, 1, 1) RVN_CASE(1, 1, 2) RVN_CASE(1, 2, 1) RVN_CASE(1, 2, 2)
#undef RVN_CASE
    }
    WgradReduce red{};
    red.part = scratch; red.dw = dw;
    red.part_stride = w.part_stride; red.S = w.S; red.KS2 = ks * ks; red.MT = w.MT; red.CT = w.CT;
    red.tiles_c = w.tiles_c; red.CO = cout; red.CI = cin; red.accumulate = accumulate ? 1 : 0;
    red.tile = 32; red.wide = w.S <= 16 ? 1 : 0;
    red.blocks = red.wide ? (w.part_stride + 255) / 256 : (w.part_stride + 31) / 32;
    if (defer) *defer = red;
    else wgrad_reduce(cx, red);
    return true;
}

}  // namespace rvn
