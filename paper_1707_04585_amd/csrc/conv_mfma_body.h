// Kernel body and argument block of the fp32 implicit-GEMM convolution (see
// conv_mfma.hip for the design), as a device function so that a launch can
// hold it next to another body.  Device code only.
#pragma once

#include "kernels.h"

namespace rvn {

struct ConvArgs {
    const float *in;      // x (forward) or upstream gradient (data gradient)
    int64_t isn, isc;
    const float *scale_shift;  // [2*CI]: a = max(in*scale + shift, 0); null = use `in` as is
    const float *w;       // [CO][CI][KS][KS] forward; [CI][CO][KS][KS] read transposed+flipped otherwise
    const float *r;       // skip operand of the epilogue (may alias out)
    int64_t rsn, rsc;
    float *out;
    int64_t osn, osc;
    int N, H, W, CI, CO;
    int ep, transposed, round_bf16;
    int TH, IMGS, bands;          // rows per band, images per workgroup, bands per image
    int trows, tcols_log2, ctl;   // pixel tile shape (trows x tcols = 16), tiles per row
    int tiles_per_img, n_tiles;   // per workgroup
    int lrows, pitch, plane, img_stride;  // LDS geometry (floats)
    int tpr_log2;                 // threads per staged row
    float inv_lrows;
    // vec32: every plane of `in`, `r`, `out` is 16-byte aligned with rows of whole 4-pixel groups, and the
    // tensors are small enough for 32-bit element offsets (below 2^30; the filter always is): staging and
    // epilogue then address with a uniform base and one 32-bit lane offset, and load unconditionally.
    // whole: every tile slot of every workgroup is a valid tile (no pixel checks in the epilogue).
    int vec32, whole;
    uint32_t m_tpi, m_ctl;        // fast-division multipliers of tiles_per_img and ctl (see fdiv_u)
    // EMIT instances (every tile slot of every workgroup a whole, valid tile): per channel and
    // wavefront the mean and centred sum of squares of the 16 * NT pixels it stores, at
    // emit[(channel * emit_tiles + workgroup * 4 + wavefront) * 2]
    float *emit;
    int emit_tiles;
};

// What a launch of the convolution needs besides its arguments.
struct ConvLaunch {
    ConvArgs a;
    int ks, kc, mt, nt;
    dim3 grid;
    size_t lds_bytes;
};

// Tiling and arguments of a convolution; false if no tiling fits.  Defined in conv_mfma.hip.
bool conv_mfma_plan(View in, const float *scale_shift, const float *w, bool transposed, int ci, int co, int ks,
                    Geo g, bool bf16, Epilogue ep, const View *r, View out, ConvLaunch &L);

namespace {

typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kConvThreads = 256;
constexpr int kWaves = 4;


__device__ __forceinline__ float bf16_round_dev(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f;
    u += 0x7fffu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xffff0000u);
}

// e / d for 0 <= e, e * d < 2^32, with m = 2^32 / d + 1 computed on the host (m = 0 stands for d = 1).
__device__ __forceinline__ int fdiv_u(int e, uint32_t m) { return m ? (int)__umulhi((uint32_t)e, m) : e; }

// Workgroup (bx, by) of the convolution; `smem` is the workgroup's dynamic LDS.
template <int KS, int MT, int NT, int KC, bool EMIT = false>
__device__ __forceinline__ void conv_mfma_f32_body(const ConvArgs &p, int bx, int by, float *smem) {
    constexpr int KS2 = KS * KS, PAD = KS / 2, LP = KS == 3 ? 4 : 0;
    constexpr int WCHUNK = (KC / 4) * KS2 * MT * 64;  // filter floats per chunk
    float *in_lds = smem;
    float *w_lds = smem + p.IMGS * p.img_stride;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int band = bx % p.bands, img_grp = bx / p.bands;
    const int n0 = img_grp * p.IMGS;
    const int row0 = band * p.TH;
    const int co0 = by * (MT * 16);
    const int HW = p.H * p.W;

    // Per-tile LDS base address of this lane's pixel (B operand) and validity.
    const int tcols = 1 << p.tcols_log2;
    const int l16 = lane & 15, kq = lane >> 4;
    const int dr = l16 >> p.tcols_log2, dc = l16 & (tcols - 1);
    int b_base[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int tile = wave + kWaves * t;
        const int img = fdiv_u(tile, p.m_tpi), rem = tile - img * p.tiles_per_img;
        const int tr = fdiv_u(rem, p.m_ctl), tc = rem - tr * p.ctl;
        b_base[t] = img * p.img_stride + kq * p.plane + (tr * p.trows + dr) * p.pitch + (LP - PAD) +
                    (tc << p.tcols_log2) + dc;
        if (tile >= p.n_tiles) b_base[t] = kq * p.plane;  // idle slot: any valid address
    }

    float4_t acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = float4_t{0.f, 0.f, 0.f, 0.f};

    const bool vec = (p.W & 3) == 0 && (p.isn & 3) == 0 && (p.isc & 3) == 0 &&
                     (reinterpret_cast<uintptr_t>(p.in) & 15) == 0;
    const int tpr = 1 << p.tpr_log2;
    const int tx = tid & (tpr - 1), ty = tid >> p.tpr_log2;
    const int rows_per_pass = kConvThreads >> p.tpr_log2;
    const int total_rows = p.IMGS * KC * p.lrows;

    // Right-hand zero quad of a staged row (3x3 only): the column just right of
    // the image must read as zero; it lies in the quad after the last data quad
    // unless W is not a multiple of 4 (then the masked tail of the data quad
    // covers it).
    const int quads = (p.W + 3) >> 2;
    const bool right_quad = KS == 3 && (p.W & 3) == 0;
    constexpr int RB = 6;                          // rows a thread loads before it stores
    constexpr int WITER = (WCHUNK + kConvThreads - 1) / kConvThreads;

    // ---- where this lane's results go: channels co0 + m*16 + 4*kq + j (j = 0..3) of
    //      its pixel.  With few accumulators the skip operand is requested now, so
    //      that it arrives under the staging and the matrix instructions (with many,
    //      the registers are not there and it is requested after them); either way
    //      it is added at the very end, with one rounding, as a separate pass would.
    //      r may alias out element for element: every address is read before the
    //      same lane writes it, and all reads come before the first write.
    constexpr bool kEarlySkip = MT * NT <= 8;
    int64_t e_off[NT];  // offset of (image, pixel) in out, -1: nothing to write
    float rv[NT][MT][4];
    // Lean form (uniform): no pixel or channel can fall outside, offsets fit 32 bits.  A result's address
    // is then a wavefront-uniform channel base plus one lane offset per tile, with no vector arithmetic
    // per access and no branch.
    const bool lean_ep = p.vec32 && p.whole && co0 + MT * 16 <= p.CO;
    uint32_t o_lane[NT], r_lane[NT];  // byte offsets
    auto locate_and_request = [&]() {
        if (lean_ep) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int tile = wave + kWaves * t;
                const int img = fdiv_u(tile, p.m_tpi), rem = tile - img * p.tiles_per_img;
                const int tr = fdiv_u(rem, p.m_ctl), tc = rem - tr * p.ctl;
                const int n = n0 + img, row = row0 + tr * p.trows + dr, col = (tc << p.tcols_log2) + dc;
                const uint32_t pix = (uint32_t)(row * p.W + col);
                o_lane[t] = ((uint32_t)n * (uint32_t)p.osn + pix + (uint32_t)(kq * 4) * (uint32_t)p.osc) * 4u;
                r_lane[t] = ((uint32_t)n * (uint32_t)p.rsn + pix + (uint32_t)(kq * 4) * (uint32_t)p.rsc) * 4u;
            }
            if (p.ep != EP_STORE) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const char *rb = reinterpret_cast<const char *>(p.r + (int64_t)(co0 + m * 16 + j) * p.rsc);  // uniform
#pragma unroll
                        for (int t = 0; t < NT; ++t) rv[t][m][j] = *reinterpret_cast<const float *>(rb + r_lane[t]);
                    }
            }
            return;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int tile = wave + kWaves * t;
            const int img = fdiv_u(tile, p.m_tpi), rem = tile - img * p.tiles_per_img;
            const int tr = fdiv_u(rem, p.m_ctl), tc = rem - tr * p.ctl;
            const int n = n0 + img, row = row0 + tr * p.trows + dr, col = (tc << p.tcols_log2) + dc;
            const bool ok = tile < p.n_tiles && n < p.N && row < p.H && row < row0 + p.TH && col < p.W;
            const int pix = row * p.W + col;
            e_off[t] = ok ? (int64_t)n * p.osn + pix : -1;
            const int64_t roff = (int64_t)n * p.rsn + pix;
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ko = co0 + m * 16 + kq * 4 + j;
                    rv[t][m][j] = p.ep != EP_STORE && ok && ko < p.CO ? p.r[roff + (int64_t)ko * p.rsc] : 0.f;
                }
        }
    };
    if (kEarlySkip) locate_and_request();

    for (int c0 = 0; c0 < p.CI; c0 += KC) {
        __syncthreads();  // previous chunk fully consumed
        // ---- filter chunk: read global memory in its own order (runs of
        //      KC*KS2 floats per output channel, or MT*16*KS2 per input channel
        //      when transposed), all loads in flight before the first store.
        float wv[WITER];
        int wdst[WITER];
        {
            // element e of the chunk is (output channel, input channel, tap) in the order of global memory:
            // the input channel is the slower index when the filter is read transposed.  Every load is
            // issued, from the filter's first element where e lies outside (the value is discarded).
            const bool tr = p.transposed != 0;
            const uint32_t s_ko = tr ? (uint32_t)KS2 : (uint32_t)p.CI * KS2, s_ch = tr ? (uint32_t)p.CO * KS2 : (uint32_t)KS2;
            const char *const wb = reinterpret_cast<const char *>(p.w);
#pragma unroll
            for (int i = 0; i < WITER; ++i) {
                const int e = tid + i * kConvThreads;
                const int o1 = e / (KC * KS2), r1 = e - o1 * (KC * KS2), i1 = r1 / KS2, t1 = r1 - i1 * KS2;
                const int o2 = e / (MT * 16 * KS2), r2 = e - o2 * (MT * 16 * KS2), i2 = r2 / KS2, t2 = r2 - i2 * KS2;
                const int kol = tr ? i2 : o1, cl = tr ? o2 : i1, t = tr ? t2 : t1;
                const int ko = co0 + kol, ch = c0 + cl;
                const bool in = e < WCHUNK && ko < p.CO && ch < p.CI;
                const uint32_t idx = (uint32_t)ko * s_ko + (uint32_t)ch * s_ch + (uint32_t)t;
                const float v = *reinterpret_cast<const float *>(wb + (in ? idx * 4u : 0u));
                wv[i] = in ? v : 0.f;
                // A-operand order; the transposed (data-gradient) filter is also flipped.
                const int tt = tr ? KS2 - 1 - t : t;
                wdst[i] = e < WCHUNK ? ((((cl >> 2) * KS2 + tt) * MT + (kol >> 4)) * 64 + (cl & 3) * 16 + (kol & 15)) : -1;
            }
        }
        // ---- input band: a = max(x*scale + shift, 0), zero outside the image
        for (int rbase = 0; rbase < total_rows; rbase += RB * rows_per_pass) {
            float4 q[RB];
            int dsti[RB];
            float sc[RB], sh[RB];
            bool live[RB];
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int rho = rbase + i * rows_per_pass + ty;
                const int pl = (int)(((float)rho + 0.5f) * p.inv_lrows);  // rho / lrows
                const int lr = rho - pl * p.lrows;
                const int img = pl / KC, c = pl - img * KC;
                const int n = n0 + img, ch = c0 + c, row = row0 - PAD + lr;
                const int col = tx * 4;
                dsti[i] = (rho < total_rows && tx < quads) ? img * p.img_stride + c * p.plane + lr * p.pitch + LP + col : -1;
                live[i] = dsti[i] >= 0 && n < p.N && ch < p.CI && row >= 0 && row < p.H;
                q[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                sc[i] = 1.f;
                sh[i] = 0.f;
                if (p.vec32) {  // (uniform) every load issued, from the tensor's first element where the item is outside
                    const uint32_t off = (uint32_t)n * (uint32_t)p.isn + (uint32_t)ch * (uint32_t)p.isc + (uint32_t)(row * p.W + col);
                    q[i] = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(p.in) + (live[i] ? off * 4u : 0u));
                    if (p.scale_shift) {
                        const uint32_t sidx = live[i] ? (uint32_t)ch * 4u : 0u;
                        sc[i] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(p.scale_shift) + sidx);
                        sh[i] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(p.scale_shift + p.CI) + sidx);
                    }
                } else if (live[i]) {
                    const float *src = p.in + (int64_t)n * p.isn + (int64_t)ch * p.isc + row * p.W + col;
                    if (vec) {
                        q[i] = *reinterpret_cast<const float4 *>(src);
                    } else {
                        q[i].x = src[0];
                        if (col + 1 < p.W) q[i].y = src[1];
                        if (col + 2 < p.W) q[i].z = src[2];
                        if (col + 3 < p.W) q[i].w = src[3];
                    }
                    if (p.scale_shift) {
                        sc[i] = p.scale_shift[ch];
                        sh[i] = p.scale_shift[p.CI + ch];
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                if (dsti[i] < 0) continue;
                float v[4] = {q[i].x, q[i].y, q[i].z, q[i].w};
                if (p.scale_shift) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = fmaxf(fmaf(v[j], sc[i], sh[i]), 0.f);
                }
                if (p.round_bf16) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = bf16_round_dev(v[j]);
                }
                if (!vec) {
                    const int col = tx * 4;
#pragma unroll
                    for (int j = 1; j < 4; ++j)
                        if (col + j >= p.W) v[j] = 0.f;
                }
                // an item outside the tensor is zero in a(x) (whatever was loaded for it)
#pragma unroll
                for (int j = 0; j < 4; ++j) v[j] = live[i] ? v[j] : 0.f;
                float *dst = in_lds + dsti[i];
                *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                if (KS == 3) {
                    if (tx == 0) *reinterpret_cast<float4 *>(dst - 4) = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (right_quad && tx == quads - 1)
                        *reinterpret_cast<float4 *>(dst + 4) = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < WITER; ++i) {
            if (wdst[i] >= 0) w_lds[wdst[i]] = p.round_bf16 ? bf16_round_dev(wv[i]) : wv[i];
        }
        __syncthreads();
        // ---- multiply
#pragma unroll
        for (int c4 = 0; c4 < KC / 4; ++c4) {
#pragma unroll
            for (int rr = 0; rr < KS; ++rr) {
#pragma unroll
                for (int ss = 0; ss < KS; ++ss) {
                    float a[MT];
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        a[m] = w_lds[((c4 * KS2 + rr * KS + ss) * MT + m) * 64 + lane];
                    const int off = c4 * 4 * p.plane + rr * p.pitch + ss;
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const float b = in_lds[b_base[t] + off];
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            acc[m][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[m], b, acc[m][t], 0, 0, 0);
                    }
                }
            }
        }
    }

    // ---- epilogue
    if (!kEarlySkip) locate_and_request();
    if (p.ep != EP_STORE) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[m][t][j] = p.ep == EP_ADD ? rv[t][m][j] + acc[m][t][j] : rv[t][m][j] - acc[m][t][j];
    }
    if (lean_ep) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                char *ob = reinterpret_cast<char *>(p.out + (int64_t)(co0 + m * 16 + j) * p.osc);  // uniform
#pragma unroll
                for (int t = 0; t < NT; ++t) *reinterpret_cast<float *>(ob + o_lane[t]) = acc[m][t][j];
            }
    } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (e_off[t] < 0) continue;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int ko = co0 + m * 16 + kq * 4 + j;
                    if (ko < p.CO) p.out[e_off[t] + (int64_t)ko * p.osc] = acc[m][t][j];
                }
            }
        }
    }
    // Statistics of what was stored, for the BN layer that reads it next: a channel's pixels of this
    // wavefront are NT registers in each of the 16 lanes of one quarter.  Sums of (v - pivot) and
    // (v - pivot)^2, pivot = the quarter's first value, are folded over the lanes four channels at a
    // time (two steps halve the channels a lane holds and add its partner's, two plain steps follow).
    if constexpr (EMIT) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            float ea[4], eb[4], piv[4];  // the pivots are uniform over the quarter
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                piv[j] = __shfl(acc[m][0][j], kq * 16, 64);
                float a = 0.f, b = 0.f;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const float d = acc[m][t][j] - piv[j];
                    a += d;
                    b += d * d;
                }
                ea[j] = a;
                eb[j] = b;
            }
            const bool up8 = (l16 & 8) != 0, up4 = (l16 & 4) != 0;
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const float keep_a = up8 ? ea[k + 2] : ea[k], send_a = up8 ? ea[k] : ea[k + 2];
                const float keep_b = up8 ? eb[k + 2] : eb[k], send_b = up8 ? eb[k] : eb[k + 2];
                ea[k] = keep_a + __shfl_xor(send_a, 8, 64);
                eb[k] = keep_b + __shfl_xor(send_b, 8, 64);
            }
            {
                const float keep_a = up4 ? ea[1] : ea[0], send_a = up4 ? ea[0] : ea[1];
                const float keep_b = up4 ? eb[1] : eb[0], send_b = up4 ? eb[0] : eb[1];
                ea[0] = keep_a + __shfl_xor(send_a, 4, 64);
                eb[0] = keep_b + __shfl_xor(send_b, 4, 64);
            }
            ea[0] += __shfl_xor(ea[0], 2, 64);
            eb[0] += __shfl_xor(eb[0], 2, 64);
            ea[0] += __shfl_xor(ea[0], 1, 64);
            eb[0] += __shfl_xor(eb[0], 1, 64);
            // the lane now holds channel j = l16 / 4 of its quarter
            const int j = l16 >> 2;
            const float pivot = j == 0 ? piv[0] : j == 1 ? piv[1] : j == 2 ? piv[2] : piv[3];
            const int ko = co0 + m * 16 + kq * 4 + j;
            if ((l16 & 3) == 0 && ko < p.CO) {
                constexpr float inv = 1.f / (16 * NT);
                const float mean = pivot + ea[0] * inv;
                const float m2 = fmaxf(eb[0] - ea[0] * ea[0] * inv, 0.f);
                float2 *dst = reinterpret_cast<float2 *>(p.emit) + (int64_t)ko * p.emit_tiles + (bx * kWaves + wave);
                *dst = make_float2(mean, m2);
            }
        }
    }
    (void)HW;
}


}  // namespace

}  // namespace rvn
