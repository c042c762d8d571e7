// The image convolution of the stem (Section 3.2: a non-reversible layer ahead
// of the reversible stages) on the matrix cores, fp32 operands.
//
// GEMM view, forward:  D[ko][pixel] = sum_k W[ko][k] * X[k][pixel], where k runs
// over the filter's taps (c, r, s) in the order they lie in memory.  One
// v_mfma_f32_16x16x4_f32 multiplies 16 output channels x 4 taps by 4 taps x 16
// output pixels.  With 3 input channels the reduction is only c_in * k * k = 27
// or 147 long, so all of it is taken tap by tap from one LDS copy of the image
// band: a lane's operand address is (offset of its tap) + (offset of its
// pixel's window), the first from a small table in LDS, the second held in a
// register per pixel tile.
//
// A workgroup (4 wavefronts) owns R output rows of one image and up to 64
// output channels.  It stages the band of input rows those windows touch, with
// the zero padding written out, and the filters of its channels in the order
// the A operand consumes them (one 16-byte read per lane and step for four
// channel tiles).  Wavefront w takes pixel tiles w*NT .. w*NT+NT-1, then
// 4*NT further on, each tile 16 consecutive pixels of the band in row-major
// order; the tiles left over after the whole rounds go one per wavefront.
// Results go to NCHW memory in 64-byte runs.
//
// Shapes whose band does not fit the LDS budget, and 1x1 filters, are left to
// the direct kernels.
#include <algorithm>

#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;
constexpr int kNT = 4;                       // pixel tiles a wavefront multiplies per filter read
constexpr size_t kLdsBudget = 96 * 1024;     // two workgroups per compute unit
constexpr size_t kBandBudget = 48 * 1024;

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int N>
struct IntC {
    static constexpr int value = N;
};

// e / d with a host-made multiplier m = 2^32 / d + 1 (exact while e * d < 2^32, which the tilings
// check; m == 0 stands for d == 1).
__device__ __forceinline__ int fast_div(int e, uint32_t m) { return m ? (int)__umulhi((uint32_t)e, m) : e; }
inline uint32_t div_magic(int d) { return d <= 1 ? 0u : (uint32_t)((1ull << 32) / (uint64_t)d + 1ull); }

// Copy `count` items into LDS with the whole workgroup: a thread requests B
// items before it stores the first, so their latencies overlap.  item(e, &tag)
// returns a valid global address for any e in [0, count) and a tag: the LDS
// index the item goes to, or its complement if zero goes there instead.
template <int B, typename Item>
__device__ __forceinline__ void stage_items(float *lds_dst, int count, Item item) {
    for (int e0 = threadIdx.x; e0 < count; e0 += B * kThreads) {
        float v[B];
        int tag[B];
#pragma unroll
        for (int u = 0; u < B; ++u) v[u] = *item(min(e0 + u * kThreads, count - 1), &tag[u]);
#pragma unroll
        for (int u = 0; u < B; ++u)
            if (e0 + u * kThreads < count) lds_dst[tag[u] < 0 ? ~tag[u] : tag[u]] = tag[u] < 0 ? 0.f : v[u];
    }
}

// The band of input rows ih0 .. ih0 + rows - 1 of every channel of image xn,
// `pad` zero columns on the left, zero outside the image: xs[c][row][LW].
__device__ __forceinline__ void stage_band(float *xs, const float *xn, int64_t xsc, const StemShape &g, int rows, int LW,
                                           uint32_t m_rows, uint32_t m_LW, int ih0, int pad) {
    stage_items<16>(xs, g.CI * rows * LW, [&](int e, int *tag) {
        const int line = fast_div(e, m_LW), cc = e - line * LW;
        const int c = fast_div(line, m_rows);
        const int ih = ih0 + (line - c * rows), iw = cc - pad;
        const int ihc = min(max(ih, 0), g.H - 1), iwc = min(max(iw, 0), g.W - 1);
        *tag = ih == ihc && iw == iwc ? e : ~e;  // inside the image, or padding
        return xn + (int64_t)c * xsc + ihc * g.W + iwc;
    });
}

struct StemTiling {
    int R;      // output rows per workgroup
    int rows;   // input rows of its band
    int LW;     // floats per band row (image row + padding on both sides)
    int bands;  // workgroups per image
    int steps;  // groups of 4 taps
    uint32_t m_rows, m_LW, m_WO;  // multipliers for fast_div
    size_t lds_bytes;
};

inline size_t band_bytes(const StemShape &g, int R) {
    const int rows = (R - 1) * g.stride + g.KS;
    const int LW = ((g.WO - 1) * g.stride + g.KS + 3) & ~3;
    return (size_t)g.CI * rows * LW * 4;
}

// false: the shape is not taken
inline bool stem_tiling(const StemShape &g, int MT, StemTiling *t) {
    if (g.KS < 3) return false;
    int R = std::max(1, std::min(g.HO, (512 + g.WO - 1) / g.WO));
    while (R > 1 && band_bytes(g, R) > kBandBudget) --R;
    t->R = R;
    t->rows = (R - 1) * g.stride + g.KS;
    t->LW = ((g.WO - 1) * g.stride + g.KS + 3) & ~3;
    t->bands = (g.HO + R - 1) / R;
    t->steps = (g.CI * g.KS * g.KS + 3) / 4;
    t->m_rows = div_magic(t->rows), t->m_LW = div_magic(t->LW), t->m_WO = div_magic(g.WO);
    t->lds_bytes = band_bytes(g, R) + (size_t)t->steps * 64 * MT * 4 + (size_t)(t->steps + 2) * 4 * 4;
    // fast_div: indices stay below the LDS size in floats, divisors below 2^15
    return t->lds_bytes <= kLdsBudget && t->LW < (1 << 15) && t->rows < (1 << 15) && g.WO < (1 << 15);
}

template <int MT>
__global__ __launch_bounds__(kThreads) void stem_conv_mfma_k(const float *__restrict__ x, int64_t xsn, int64_t xsc,
                                                             const float *__restrict__ w, float *__restrict__ out,
                                                             int64_t osn, int64_t osc, StemShape g, StemTiling tl) {
    extern __shared__ __align__(16) float lds[];
    const int taps = g.CI * g.KS * g.KS, pad = (g.KS - 1) / 2;
    const int band_floats = g.CI * tl.rows * tl.LW;  // a multiple of 4
    float *xs = lds;                                 // [CI][rows][LW]
    float *wl = xs + band_floats;                    // [steps][64 lanes][MT]
    int *toff = reinterpret_cast<int *>(wl + tl.steps * 64 * MT);  // [(steps + 2) * 4]
    const int n = blockIdx.x / tl.bands, band = blockIdx.x - n * tl.bands;
    const int p0 = band * tl.R;
    const int k0 = blockIdx.y * (16 * MT);
    const int tid = threadIdx.x;

    // ---- the band: image rows p0*stride - pad .. of every input channel, zero outside the image
    stage_band(xs, x + (int64_t)n * xsn, xsc, g, tl.rows, tl.LW, tl.m_rows, tl.m_LW, p0 * g.stride - pad, pad);
    // ---- the filters: wl[(step * 64 + lane) * MT + mt] = w[k0 + 16 mt + lane % 16][4 step + lane / 16]
    stage_items<16>(wl, tl.steps * 64 * MT, [&](int e, int *tag) {
        const int mt = e % MT, ln = (e / MT) & 63, step = e / (MT * 64);
        const int row = k0 + 16 * mt + (ln & 15), tap = 4 * step + (ln >> 4);
        const bool ok = row < g.CO && tap < taps;
        *tag = ok ? e : ~e;
        return w + (ok ? (int64_t)row * taps + tap : 0);
    });
    // ---- where tap t = (c, r, s) lies relative to a window's first element
    for (int t = tid; t < (tl.steps + 2) * 4; t += kThreads) {
        const int c = t / (g.KS * g.KS), rs = t - c * g.KS * g.KS;
        const int r = rs / g.KS, s = rs - r * g.KS;
        toff[t] = t < taps ? (c * tl.rows + r) * tl.LW + s : 0;
    }
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kq = lane >> 4;
    const int rows_here = min(tl.R, g.HO - p0);
    const int npix = rows_here * g.WO, tiles = (npix + 15) / 16;
    // NT consecutive tiles from t0 on: all taps, then the stores
    auto run_tiles = [&](auto nt_tag, int t0) {
        constexpr int NT = decltype(nt_tag)::value;
        int pixbase[NT];
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int pix = min((t0 + i) * 16 + l16, npix - 1);  // slots past the end repeat the last pixel
            const int pr = fast_div(pix, tl.m_WO), q = pix - pr * g.WO;
            pixbase[i] = pr * g.stride * tl.LW + q * g.stride;
        }
        f32x4 acc[MT][NT];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int i = 0; i < NT; ++i) acc[m][i] = f32x4{0.f, 0.f, 0.f, 0.f};
        // The operands of step + 1 (and the tap offset of step + 2) are requested before the
        // instructions of step are issued, so the LDS latency runs behind the matrix pipe.
        auto load_a = [&](int step, float(&a)[MT]) {
            const float *ap = wl + (step * 64 + lane) * MT;  // MT * 4 bytes, aligned to that
            if constexpr (MT == 4) {
                const f32x4 av = *reinterpret_cast<const f32x4 *>(ap);
                a[0] = av[0], a[1] = av[1], a[2] = av[2], a[3] = av[3];
            } else {
                const float2 av = *reinterpret_cast<const float2 *>(ap);
                a[0] = av.x, a[1] = av.y;
            }
        };
        float a_cur[MT], b_cur[NT];
        int to_nxt = toff[4 + kq];  // the table has two steps of zeros behind the last
        {
            const int to = toff[kq];
            load_a(0, a_cur);
#pragma unroll
            for (int i = 0; i < NT; ++i) b_cur[i] = xs[to + pixbase[i]];
        }
        for (int step = 0; step < tl.steps; ++step) {
            float a_nxt[MT], b_nxt[NT];
            load_a(min(step + 1, tl.steps - 1), a_nxt);
#pragma unroll
            for (int i = 0; i < NT; ++i) b_nxt[i] = xs[to_nxt + pixbase[i]];
            to_nxt = toff[(step + 2) * 4 + kq];
            const bool live = step * 4 + kq < taps;  // the filter is zero there; keep the product finite
#pragma unroll
            for (int i = 0; i < NT; ++i) b_cur[i] = live ? b_cur[i] : 0.f;
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int i = 0; i < NT; ++i)
                    acc[m][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[m], b_cur[i], acc[m][i], 0, 0, 0);
#pragma unroll
            for (int m = 0; m < MT; ++m) a_cur[m] = a_nxt[m];
#pragma unroll
            for (int i = 0; i < NT; ++i) b_cur[i] = b_nxt[i];
        }
        // lane's results: channels k0 + 16 m + 4 kq + j (j = 0..3) of pixel l16 of each tile
#pragma unroll
        for (int i = 0; i < NT; ++i) {
            const int pix = (t0 + i) * 16 + l16;
            if (pix >= npix) continue;
            const int pr = pix / g.WO, q = pix - pr * g.WO;
            float *o = out + (int64_t)n * osn + (int64_t)(p0 + pr) * g.WO + q;
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ch = k0 + 16 * m + 4 * kq + j;
                    if (ch < g.CO) o[(int64_t)ch * osc] = acc[m][i][j];
                }
        }
    };
    // whole rounds of kNT tiles per wavefront, then the rest one tile per wavefront and round
    const int full = tiles / (4 * kNT) * (4 * kNT);
    for (int t0 = wave * kNT; t0 < full; t0 += 4 * kNT) run_tiles(IntC<kNT>{}, t0);
    for (int t = full + wave; t < tiles; t += 4) run_tiles(IntC<1>{}, t);
}

template <int MT>
bool launch_fwd(Ctx &cx, View x, const float *w, const StemShape &g, View out) {
    StemTiling tl;
    if (!stem_tiling(g, MT, &tl)) return false;
    static bool raised = false;  // more than 64 KB of dynamic LDS has to be asked for once
    if (!raised) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(stem_conv_mfma_k<MT>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
        if (e != hipSuccess) {
            cx.fail(e);
            return true;
        }
        raised = true;
    }
    const dim3 grid((unsigned)(g.N * tl.bands), (unsigned)((g.CO + 16 * MT - 1) / (16 * MT)));
    cx.run(stem_conv_mfma_k<MT>, grid, dim3(kThreads), tl.lds_bytes, (const float *)x.p, x.sn, x.sc, w, out.p, out.sn,
           out.sc, g, tl);
    return true;
}

// ---------------------------------------------------------------------------
// Filter gradient:  dW[ko][k] = sum over output pixels of dh[ko][pixel] * X[k][pixel],
// pixels on the reduction side.  One instruction multiplies 16 output channels
// x 4 pixels (A, from an LDS copy of dh) by 4 pixels x 16 taps (B, from the LDS
// band, address = tap offset held in a register per tap tile + window offset of
// the pixel).  A workgroup owns 64 output channels and a run of consecutive
// (image, band) units; wavefront w multiplies all four channel tiles by the tap tiles w,
// w + 4, ... (so a B operand is read by one wavefront only); the sums stay in
// registers over the whole run and are written once, as partial result
// part[chunk][ko][tap]; stem_wgrad_reduce_k adds the chunks in order.
// ---------------------------------------------------------------------------
struct StemWgradTiling {
    int R, rows, LW, bands;
    int chunks;  // workgroups per 64 output channels: each takes upc consecutive (image, band) units
    int upc;
    int PP;   // pixel pitch of the dh copy: = 4 mod 64, so 16 channels x 4 pixels fall into 64 banks
    int ntw;  // tap tiles of 16 per wavefront (1..4)
    uint32_t m_rows, m_LW, m_WO;  // multipliers for fast_div
    uint32_t m_bands;  // 0: divide
    int npad_full;     // pixels of a full band, rounded up to 4, and its multiplier (npad_full > 1)
    uint32_t m_npad;
    size_t lds_bytes;
};

inline bool stem_wgrad_tiling(const StemShape &g, StemWgradTiling *t) {
    if (g.KS < 3) return false;
    const int taps = g.CI * g.KS * g.KS;
    if (taps > 256) return false;
    const int R = std::max(1, std::min(g.HO, 128 / g.WO));
    t->R = R;
    t->rows = (R - 1) * g.stride + g.KS;
    t->LW = ((g.WO - 1) * g.stride + g.KS + 3) & ~3;
    t->bands = (g.HO + R - 1) / R;
    const int groups = (g.CO + 63) / 64;
    const int64_t units = (int64_t)g.N * t->bands;
    if (units >= (1 << 30)) return false;
    int64_t chunks = std::max(1, 768 / groups);                    // about three workgroups per compute unit,
    chunks = std::min(chunks, std::max<int64_t>(64, units / 4));   // but few partial results for small jobs
    chunks = std::min(chunks, units);
    t->upc = (int)((units + chunks - 1) / chunks);
    t->chunks = (int)((units + t->upc - 1) / t->upc);  // no empty chunk
    const int npad = (R * g.WO + 3) & ~3;
    t->PP = ((npad - 4 + 63) / 64) * 64 + 4;
    t->npad_full = npad, t->m_npad = div_magic(npad);
    t->m_bands = units * t->bands < (1ll << 32) ? div_magic(t->bands) : 0u;
    t->ntw = ((taps + 15) / 16 + 3) / 4;
    t->m_rows = div_magic(t->rows), t->m_LW = div_magic(t->LW), t->m_WO = div_magic(g.WO);
    t->lds_bytes = band_bytes(g, R) + (size_t)64 * t->PP * 4;
    return t->lds_bytes <= kLdsBudget && t->LW < (1 << 15) && t->rows < (1 << 15) && g.WO < (1 << 15);
}

template <int NTW>
__global__ __launch_bounds__(kThreads) void stem_wgrad_mfma_k(const float *__restrict__ x, int64_t xsn, int64_t xsc,
                                                              const float *__restrict__ dh, int64_t dsn, int64_t dsc,
                                                              float *__restrict__ part, StemShape g, StemWgradTiling tl) {
    extern __shared__ __align__(16) float lds[];
    const int taps = g.CI * g.KS * g.KS, pad = (g.KS - 1) / 2;
    const int band_floats = g.CI * tl.rows * tl.LW;
    float *xs = lds;                // [CI][rows][LW]
    float *dl = xs + band_floats;   // [64][PP]
    const int k0 = blockIdx.y * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kq = lane >> 4;

    // this wavefront's tap tiles: wave, wave + 4, ...; where the lane's tap of each lies relative to
    // a window's first element (tiles and taps past the last are multiplied like the others and never stored)
    int to[NTW];
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
        const int t = 16 * (wave + 4 * i) + l16;
        const int c = t / (g.KS * g.KS), rs = t - c * g.KS * g.KS;
        const int r = rs / g.KS, s = rs - r * g.KS;
        to[i] = t < taps ? (c * tl.rows + r) * tl.LW + s : 0;
    }
    f32x4 acc[4][NTW];
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int i = 0; i < NTW; ++i) acc[m][i] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int u0 = blockIdx.x * tl.upc, u1 = min(g.N * tl.bands, u0 + tl.upc);
    for (int u = u0; u < u1; ++u) {
        const int n = tl.bands == 1 ? u : (tl.m_bands ? fast_div(u, tl.m_bands) : u / tl.bands);
        const int band = u - n * tl.bands;
        const float *xn = x + (int64_t)n * xsn;
        const float *dn = dh + (int64_t)n * dsn;
        const int p0 = band * tl.R;
        const int rows_here = min(tl.R, g.HO - p0);
        const int npix = rows_here * g.WO, npad = (npix + 3) & ~3;
        __syncthreads();  // the previous band has been read
        stage_band(xs, xn, xsc, g, tl.rows, tl.LW, tl.m_rows, tl.m_LW, p0 * g.stride - pad, pad);
        // dh of the band's pixels, 64 channels; zero past the last channel and the last pixel
        {
            const uint32_t m_npad = npad == tl.npad_full ? tl.m_npad : 0u;
            stage_items<16>(dl, 64 * npad, [&](int e, int *tag) {
                const int ch = m_npad ? fast_div(e, m_npad) : e / npad, pix = e - ch * npad;
                const int dst = ch * tl.PP + pix;
                *tag = k0 + ch < g.CO && pix < npix ? dst : ~dst;
                return dn + (int64_t)min(k0 + ch, g.CO - 1) * dsc + (int64_t)p0 * g.WO + min(pix, npix - 1);
            });
        }
        __syncthreads();
        // operands of one step: dh of 4 pixels x 16 channels per channel tile, the image at the
        // wavefront's taps of those pixels' windows; step + 1 is requested before step is multiplied
        const float *ap = dl + l16 * tl.PP + kq;
        auto operands = [&](int step, float(&a)[4], float(&b)[NTW]) {
            const int pc = min(4 * step + kq, npix - 1);
            const int pr = fast_div(pc, tl.m_WO), q = pc - pr * g.WO;
            const int pb = pr * g.stride * tl.LW + q * g.stride;
#pragma unroll
            for (int m = 0; m < 4; ++m) a[m] = ap[m * 16 * tl.PP + 4 * step];
#pragma unroll
            for (int i = 0; i < NTW; ++i) b[i] = xs[to[i] + pb];
        };
        const int nsteps = npad / 4;
        float a_cur[4], b_cur[NTW];
        operands(0, a_cur, b_cur);
        for (int step = 0; step < nsteps; ++step) {
            float a_nxt[4], b_nxt[NTW];
            operands(min(step + 1, nsteps - 1), a_nxt, b_nxt);
            const bool live = 4 * step + kq < npix;  // dh is zero there; keep the product finite
#pragma unroll
            for (int i = 0; i < NTW; ++i) b_cur[i] = live ? b_cur[i] : 0.f;
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int i = 0; i < NTW; ++i)
                    acc[m][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[m], b_cur[i], acc[m][i], 0, 0, 0);
#pragma unroll
            for (int m = 0; m < 4; ++m) a_cur[m] = a_nxt[m];
#pragma unroll
            for (int i = 0; i < NTW; ++i) b_cur[i] = b_nxt[i];
        }
    }
    // lane's sums: channels k0 + 16 m + 4 kq + j, tap 16 (wave + 4 i) + l16
    float *o = part + (int64_t)blockIdx.x * g.CO * taps;
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
        const int t = 16 * (wave + 4 * i) + l16;
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ko = k0 + 16 * m + 4 * kq + j;
                if (ko < g.CO && t < taps) o[(int64_t)ko * taps + t] = acc[m][i][j];
            }
    }
}

template <int NTW>
void launch_wgrad(Ctx &cx, View x, View dh, const StemShape &g, const StemWgradTiling &tl, float *part) {
    static bool raised = false;
    if (!raised) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(stem_wgrad_mfma_k<NTW>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBudget);
        if (e != hipSuccess) {
            cx.fail(e);
            return;
        }
        raised = true;
    }
    const dim3 grid((unsigned)tl.chunks, (unsigned)((g.CO + 63) / 64));
    cx.run(stem_wgrad_mfma_k<NTW>, grid, dim3(kThreads), tl.lds_bytes, (const float *)x.p, x.sn, x.sc,
           (const float *)dh.p, dh.sn, dh.sc, part, g, tl);
}

}  // namespace

bool stem_conv_mfma_takes(const StemShape &g) {
    StemTiling tl;
    return stem_tiling(g, g.CO <= 32 ? 2 : 4, &tl);
}

void stem_conv_mfma(Ctx &cx, View x, const float *w, const StemShape &g, View out) {
    if (g.CO <= 32)
        launch_fwd<2>(cx, x, w, g, out);
    else
        launch_fwd<4>(cx, x, w, g, out);
}

int stem_wgrad_mfma_chunks(const StemShape &g) {
    StemWgradTiling tl;
    return stem_wgrad_tiling(g, &tl) ? tl.chunks : 0;
}

void stem_wgrad_mfma(Ctx &cx, View x, View dh, const StemShape &g, float *part) {
    StemWgradTiling tl;
    if (!stem_wgrad_tiling(g, &tl)) {
        cx.fail(hipErrorInvalidValue);  // the caller asks stem_wgrad_mfma_chunks first
        return;
    }
    switch (tl.ntw) {
        case 1: launch_wgrad<1>(cx, x, dh, g, tl, part); break;
        case 2: launch_wgrad<2>(cx, x, dh, g, tl, part); break;
        case 3: launch_wgrad<3>(cx, x, dh, g, tl, part); break;
        default: launch_wgrad<4>(cx, x, dh, g, tl, part); break;
    }
}

}  // namespace rvn
