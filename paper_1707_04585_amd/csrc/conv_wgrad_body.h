// Kernel body and argument block of the fp32 filter-gradient kernel (see
// conv_wgrad.hip for the design), as a device function so that a launch can
// hold it next to another body.  Device code only.
#pragma once

#include "kernels.h"

namespace rvn {

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

// What a launch of the filter gradient needs besides its arguments.
struct WgradLaunch {
    WgradArgs a;
    int ks, mt, ct;
    bool vec;
    dim3 grid;
    size_t lds_bytes;
};

// Plan and arguments of a filter gradient and of the ordered sum that follows it; false if no
// plan fits.  Defined in conv_wgrad.hip.
bool conv_wgrad_plan(View x, const float *scale_shift, bool bf16, View dh, int cin, int cout, int ks, Geo g,
                     float *scratch, float *dw, bool accumulate, WgradLaunch &L, WgradReduce &red);

namespace {

typedef float wg_float4_t __attribute__((ext_vector_type(4)));

constexpr int kWgradThreads = 256;
constexpr int kItemsA = 8, kItemsD = 5;  // 16-byte LDS items of a / of dh a thread stages per unit (at most)


// e / d for 0 <= e, e * d < 2^32, with m = 2^32 / d + 1 computed on the host
// (m = 0 stands for d = 1).
__device__ __forceinline__ int fdiv(int e, uint32_t m) { return m ? (int)__umulhi((uint32_t)e, m) : e; }

__device__ __forceinline__ float bf16_round_wg(float f) {
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

// Workgroup (bx, by, bz) of a grid that is gz deep; `smem` is the workgroup's dynamic LDS.
template <int KS, int MT, int CT, bool VEC>
__device__ __forceinline__ void conv_wgrad_mfma_body(const WgradArgs &p, int bx, int by, int bz, int gz, float *smem) {
    constexpr int KS2 = KS * KS, PAD = KS / 2, LP = KS == 3 ? 4 : 0;
    constexpr int WT = MT * CT, KW = 4 / WT;  // tile owners, pixel shares
    static_assert(WT == 1 || WT == 2 || WT == 4, "one tile per wavefront");
    float *a_lds = smem;
    float *d_lds = smem + CT * 16 * p.a_plane;
    __shared__ float ss_lds[2 * CT * 16];  // scale, shift of this workgroup's input channels

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ko0 = by * (MT * 16), c0 = bz * (CT * 16);
    const int u_begin = bx * p.upw;
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
            const int e = tid + i * kWgradThreads;
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
            const int e = tid + i * kWgradThreads;
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
                    if (round_bf16) v[j] = bf16_round_wg(v[j]);
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
                for (int j = 0; j < 4; ++j) v[j] = bf16_round_wg(v[j]);
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

    wg_float4_t acc[KS2];
#pragma unroll
    for (int t = 0; t < KS2; ++t) acc[t] = wg_float4_t{0.f, 0.f, 0.f, 0.f};

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
    float *out = p.part + (int64_t)bx * p.part_stride + (int64_t)(by * gz + bz) * (WT * KS2 * 256);
    for (int idx = tid; idx < WT * KS2 * 256; idx += kWgradThreads) {
        const int tl = idx / (KS2 * 256), rest = idx - tl * (KS2 * 256);
        float v = red[(tl * KW) * KS2 * 256 + rest];
#pragma unroll
        for (int k = 1; k < KW; ++k) v += red[(tl * KW + k) * KS2 * 256 + rest];
        out[idx] = v;
    }
}


}  // namespace

}  // namespace rvn
