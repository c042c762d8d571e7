// Kernel body and argument block of the 3x3 convolution with bf16 operands (see
// conv3x3_bf16.hip for the design), as a device function so that a launch can
// hold it next to another body.  Device code only.
#pragma once

#include <type_traits>

#include "kernels.h"
#include "stats_fold.h"

namespace rvn {

struct C3Args {
    const float *in;  // x (forward) or upstream gradient (data gradient), fp32 NCHW planes
    int64_t isn, isc;
    const float *scale_shift;  // [2*CI]: a = max(in*scale + shift, 0); null = use `in` as is
    const uint16_t *wq;        // filter in bf16, [CO][9][CIP]
    int CIP;
    const float *r;  // skip operand of the epilogue (may alias out)
    int64_t rsn, rsc;
    float *out;
    int64_t osn, osc;
    int N, H, W, CI, CO, ep;
    int stride;           // 1, or 2 (H and W even): only every second row and column of the result exists, OH = H / 2, OW = W / 2
    int TR, IMGS, bands;  // rows and images per pixel block, blocks per image column
    int pix_per_img;      // TR * W
    int n_pix;            // IMGS * TR * W
    int lrows, lcols;     // LDS tile: TR + 2 rows, W + 2 columns
    int q_per_img;        // quads of the widest band range: ceil((TR + 2) * W / 4)
    int in_items;         // IMGS * q_per_img * (KC / 8)
    int wg_x, wg_x8;      // pixel blocks in all; the launch's ids along x (wg_x rounded up to a multiple of 8)
    int chunks, cps;      // channel chunks in total and per split
    float *part;          // partial tiles [split][n][ko][h*w] when gridDim.z > 1
    int64_t part_stride;
    // EMIT instances (no split, every pixel slot of every workgroup a valid pixel): per channel and
    // wavefront the mean and centred sum of squares of the 32 * NTW pixels it stores, at
    // emit[(channel * emit_tiles + blockIdx.x * WN + wn) * 2]
    float *emit;
    int emit_tiles;
};

// What a launch of the convolution needs besides its arguments.  S > 1: the input channels are split
// over the grid's z, partial tiles go to scratch and conv3x3_bf16_finish sums them.
struct C3Launch {
    C3Args a;
    int MTW, KC, NI, S;
    dim3 grid;
    size_t lds_bytes;
    const float *scratch;
};

// Tiling and arguments of a 3x3 convolution without epilogue statistics; false if the kernel does not
// take the layer.  Defined in conv3x3_bf16.hip.
bool conv3x3_bf16_plan(View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g, Epilogue ep,
                       const View *r, View out, float *scratch, C3Launch &L, int stride = 1);
// The launch that sums the partial tiles of a split convolution (nothing to do when L.S == 1); g: the
// geometry of the result.
void conv3x3_bf16_finish(Ctx &cx, const C3Launch &L, Geo g);

namespace {

namespace c3 {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef float f4u_t __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u2u_t __attribute__((ext_vector_type(2), aligned(4)));  // four bf16, only element aligned

constexpr int kThreads = 256;
constexpr int kPadK = 8;     // bf16 elements of padding per LDS record
constexpr int kInItems = 2;  // activation staging items per thread and chunk, at most


__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const float2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<const uint32_t *>(&b);
}

// Buffer resource over `bytes` bytes at `base` (raw, no stride, dword data): accesses through it take a
// 32-bit per-lane byte offset and a 32-bit wavefront-uniform byte offset from scalar registers, so no
// vector instruction is spent on addresses.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_over(const void *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}

// WM x WN wavefronts (WM * WN = 4), each MTW x NTW tiles of 32 output channels
// x 32 pixels; KC input channels per chunk.  NI: activation staging items per
// thread and chunk.  With NI == 1 the activation loads run two chunks ahead of the
// matrix instructions (two register sets): a chunk's matrix work is well below one
// memory round trip, so with one chunk of lookahead every chunk paid for one.
// IN16: `in` holds bf16 already (dense planes, same element strides; no BN prologue): the values a
// conversion on load would produce, so results are the same bits at half the bytes.
template <int WM, int MTW, int NTW, int KC, bool EMIT = false, int NI = kInItems, bool IN16 = false>
__device__ __forceinline__ void conv3x3_bf16_body(const C3Args &p, int bx_launch, int by, int bz, int gz, uint16_t *smem16) {
    constexpr int WN = 4 / WM;
    constexpr int REC = KC + kPadK, OCTS = KC / 8;
    constexpr int CH = WM * MTW * 32;  // output channels per workgroup
    constexpr int W_ITEMS = CH * 9 * OCTS, W_PER = (W_ITEMS + kThreads - 1) / kThreads;
    uint16_t *in_lds = smem16;                                    // [IMGS][lrows][lcols][REC]
    uint16_t *w_lds = smem16 + p.IMGS * p.lrows * p.lcols * REC;  // [CH][9][REC]
    float *ss_lds = reinterpret_cast<float *>(w_lds + CH * 9 * REC);  // [2][CI]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    // Workgroup ids go round-robin over the 8 dies; give every die a contiguous range of pixel blocks
    // (the launch has a multiple of 8 ids along x), so that neighbouring bands, which share two of their
    // six input rows, find them in the same L2.
    // (Only where an image is cut into bands; whole-image blocks share nothing and keep the launch order:
    // remapped, the 32x32-and-smaller layers measured 4 % slower.)
    const int bx = p.bands > 1 ? (bx_launch & 7) * (p.wg_x8 >> 3) + (bx_launch >> 3) : bx_launch;
    if (bx >= p.wg_x) return;
    const int band = bx % p.bands, img_grp = bx / p.bands;
    const int n0 = img_grp * p.IMGS, row0 = band * p.TR;  // (row0, TR, bands: rows of the result)
    const int st = p.stride, OH = p.H / st, OW = p.W / st;
    const int co0 = by * CH;
    const int N = p.N, H = p.H, W = p.W, CI = p.CI, CO = p.CO;
    const int l32 = lane & 31, kg = lane >> 5;
    const bool bn = p.scale_shift != nullptr;
    constexpr int kInBytes = IN16 ? 2 : 4;

    // ---- zero the activation tile once (halo, rows outside the image, unused
    //      slots stay zero) and fetch scale/shift
    {
        const int n16 = p.IMGS * p.lrows * p.lcols * REC / 8;
        for (int e = tid; e < n16; e += kThreads) reinterpret_cast<uint4_t *>(in_lds)[e] = uint4_t{0u, 0u, 0u, 0u};
        if (bn)
            for (int e = tid; e < 2 * CI; e += kThreads) ss_lds[e] = p.scale_shift[e];
    }

    // ---- this thread's activation items: (image, quad of the band's pixel range, channel octet)
    const int in_row0 = st * row0 - 1;  // the input row of the tile's first row
    const int start_row = max(0, in_row0), end_row = min(H, st * (row0 + p.TR - 1) + 2);
    const int range = (end_row - start_row) * W;  // contiguous pixels of the plane this block reads
    uint32_t it_off[NI];                          // byte offset of (image, pixel) in a plane (dead items: 0)
    int it_rec[NI], it_info[NI];                  // LDS record of pixel 0; col | nvalid << 16 | oc << 24
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int e = tid + i * kThreads;
        const int oc = e % OCTS, t = e / OCTS;
        const int q = t % p.q_per_img, img = t / p.q_per_img;
        const int n = n0 + img, start = 4 * q;
        const bool live = e < p.in_items && n < N && start < range;
        // the last quad of the range is moved back to end with it: the pixels it shares
        // with its neighbour are written twice, with the same values
        const int ld = min(start, range - 4);
        const int lin = start_row * W + ld, row = lin / W, col = lin - row * W;
        it_off[i] = live ? (uint32_t)(((int64_t)n * p.isn + start_row * W + ld) * kInBytes) : 0u;
        it_rec[i] = (img * p.lrows + (row - in_row0)) * p.lcols + 1 + col;
        const int nvalid = live ? 4 : 0;
        it_info[i] = col | (nvalid << 16) | (oc << 24);
    }

    // ---- this lane's pixel in each of its NTW pixel groups
    int b_rec[NTW], o_img[NTW], o_pix[NTW];
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        const int f = (wn * NTW + t) * 32 + l32;
        const int img = f / p.pix_per_img, rem = f - img * p.pix_per_img;
        const int rr = rem / OW, cc = rem - rr * OW;
        const bool ok = f < p.n_pix && n0 + img < N && row0 + rr < OH;
        b_rec[t] = f < p.n_pix ? (img * p.lrows + st * rr) * p.lcols + st * cc : 0;
        o_img[t] = ok ? n0 + img : -1;
        o_pix[t] = (row0 + rr) * OW + cc;
    }

    float16_t acc[MTW][NTW];
#pragma unroll
    for (int m = 0; m < MTW; ++m)
#pragma unroll
        for (int t = 0; t < NTW; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][t][i] = 0.f;

    // register sets of activation loads (with bf16 input four half-size sets, four chunks ahead, measured the
    // same as two: in the shared gradient launch the filter gradient is the longer part)
    constexpr int SETS = NI == 1 ? 2 : 1;
    using Quad = typename std::conditional<IN16, u2u_t, f4u_t>::type;  // four pixels of one channel as loaded
    Quad gin[SETS][NI][8];
    uint4_t gw[W_PER];
    const char *const in_base = reinterpret_cast<const char *>(p.in);
    const int64_t isc_b = p.isc * kInBytes;

    // global -> registers: the activations of chunk c0 into register set `set`, the filter of chunk c0
    auto g2r_act = [&](Quad (&g)[NI][8], int c0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int oc = it_info[i] >> 24;
            // octets past the last channel read the chunk's first octet instead and are zeroed later
            const uint32_t off = it_off[i] + (c0 + oc * 8 < CI ? (uint32_t)(oc * 8 * isc_b) : 0u);
#pragma unroll
            for (int k = 0; k < 8; ++k)
                g[i][k] = *reinterpret_cast<const Quad *>(in_base + (int64_t)(c0 + k) * isc_b + off);
        }
    };
    auto g2r_w = [&](int c0) {
#pragma unroll
        for (int i = 0; i < W_PER; ++i) {
            const int e = tid + i * kThreads;
            const int oc = e % OCTS, t = e / OCTS;
            const bool ok = e < W_ITEMS && co0 + t / 9 < CO && c0 + oc * 8 < p.CIP;
            gw[i] = *reinterpret_cast<const uint4_t *>(p.wq + (ok ? ((int64_t)co0 * 9 + t) * p.CIP + c0 + oc * 8 : 0));
            if (!ok) gw[i] = uint4_t{0u, 0u, 0u, 0u};
        }
    };
    // registers -> LDS: BN + ReLU + rounding of the activations of chunk c0; the filter as loaded
    auto r2l_act = [&](const Quad (&g)[NI][8], int c0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int info = it_info[i];
            const int col = info & 0xffff, nvalid = (info >> 16) & 15, oc = info >> 24;
            if (nvalid == 0) continue;
            const bool chan_ok = c0 + oc * 8 < CI;
            if constexpr (IN16) {
                // dword w of channel k holds pixels 2w, 2w + 1; a record wants, per pixel, the channels in
                // pairs: one byte permute per dword (low halves for even pixels, high halves for odd ones)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int rec = it_rec[i] + j + (col + j >= W ? 2 : 0);
                    const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
                    uint4_t q;
#pragma unroll
                    for (int d = 0; d < 4; ++d) {
                        const uint32_t pr = __builtin_amdgcn_perm(g[i][2 * d + 1][j >> 1], g[i][2 * d][j >> 1], sel);
                        q[d] = chan_ok ? pr : 0u;
                    }
                    *reinterpret_cast<uint4_t *>(in_lds + rec * REC + oc * 8) = q;
                }
                continue;
            } else {
            float v[8][4];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const f4u_t x = g[i][k];
                float x0 = x[0], x1 = x[1], x2 = x[2], x3 = x[3];
                if (bn) {
                    const int ch = chan_ok ? c0 + oc * 8 + k : 0;
                    const float sc = ss_lds[ch], sh = ss_lds[CI + ch];
                    x0 = fmaxf(fmaf(x0, sc, sh), 0.f);
                    x1 = fmaxf(fmaf(x1, sc, sh), 0.f);
                    x2 = fmaxf(fmaf(x2, sc, sh), 0.f);
                    x3 = fmaxf(fmaf(x3, sc, sh), 0.f);
                }
                v[k][0] = chan_ok ? x0 : 0.f;
                v[k][1] = chan_ok ? x1 : 0.f;
                v[k][2] = chan_ok ? x2 : 0.f;
                v[k][3] = chan_ok ? x3 : 0.f;
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // pixels past the end of an image row continue in the next tile row, after 2 halo records
                const int rec = it_rec[i] + j + (col + j >= W ? 2 : 0);
                const uint4_t q = {pack2(v[0][j], v[1][j]), pack2(v[2][j], v[3][j]), pack2(v[4][j], v[5][j]),
                                   pack2(v[6][j], v[7][j])};
                *reinterpret_cast<uint4_t *>(in_lds + rec * REC + oc * 8) = q;
            }
            }
        }
    };
    auto r2l_w = [&]() {
#pragma unroll
        for (int i = 0; i < W_PER; ++i) {
            const int e = tid + i * kThreads;
            if (e < W_ITEMS) *reinterpret_cast<uint4_t *>(w_lds + (e / OCTS) * REC + (e % OCTS) * 8) = gw[i];
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int rr = 0; rr < 3; ++rr) {
#pragma unroll
            for (int ss = 0; ss < 3; ++ss) {
#pragma unroll
                for (int ks = 0; ks < KC / 16; ++ks) {
                    bf16x8_t a[MTW], b[NTW];
#pragma unroll
                    for (int m = 0; m < MTW; ++m)
                        a[m] = *reinterpret_cast<const bf16x8_t *>(
                            w_lds + (((wm * MTW + m) * 32 + l32) * 9 + rr * 3 + ss) * REC + ks * 16 + kg * 8);
#pragma unroll
                    for (int t = 0; t < NTW; ++t)
                        b[t] = *reinterpret_cast<const bf16x8_t *>(
                            in_lds + (b_rec[t] + rr * p.lcols + ss) * REC + ks * 16 + kg * 8);
#pragma unroll
                    for (int m = 0; m < MTW; ++m)
#pragma unroll
                        for (int t = 0; t < NTW; ++t)
                            acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], b[t], acc[m][t], 0, 0, 0);
                }
            }
        }
    };

    const int chunk0 = bz * p.cps, chunk1 = min(p.chunks, chunk0 + p.cps);
    g2r_w(chunk0 * KC);
    g2r_act(gin[0], chunk0 * KC);
#pragma unroll
    for (int st = 1; st < SETS; ++st)
        if (chunk0 + st < chunk1) g2r_act(gin[st], (chunk0 + st) * KC);
    __syncthreads();  // tile zeroed, scale/shift in LDS
    r2l_w();
    r2l_act(gin[0], chunk0 * KC);
    __syncthreads();
    // LDS holds chunk ch, which came from register set st; that set is free and takes the loads of chunk
    // ch + SETS, the chunks in between are in flight in the other sets.  The filter (small, cached) keeps
    // one chunk of lookahead and is requested before the activations, so that waiting for it does not
    // wait for them.
    for (int base = chunk0; base < chunk1; base += SETS) {
#pragma unroll
        for (int st = 0; st < SETS; ++st) {
            const int ch = base + st;
            if (ch >= chunk1) break;
            if (ch + 1 < chunk1) g2r_w((ch + 1) * KC);
            if (ch + SETS < chunk1) g2r_act(gin[st], (ch + SETS) * KC);
            multiply();
            if (ch + 1 < chunk1) {
                __syncthreads();  // every wavefront has read chunk ch
                r2l_w();
                r2l_act(gin[(st + 1) % SETS], (ch + 1) * KC);
                __syncthreads();
            }
        }
    }

    // ---- epilogue: register i of a lane is channel 8*(i/4) + 4*kg + i%4 of its pixel.
    //      Every access is a buffer access: a 32-bit per-lane byte offset (image, pixel, 4*kg channels)
    //      plus a wavefront-uniform byte offset (the channel without the lane's 4*kg) that lives in scalar
    //      registers; the host keeps every tensor handed to one launch below 4 GB.  With a 64-bit address
    //      per lane and access, address arithmetic was half of the kernel's vector instructions.
    const bool partial = gz > 1;
    const uint32_t HW4 = (uint32_t)(OH * OW) * 4u;
    const uint32_t osc4 = (uint32_t)p.osc * 4u, rsc4 = (uint32_t)p.rsc * 4u;
    const __amdgpu_buffer_rsrc_t out_rs = partial ? buffer_over(p.part + bz * p.part_stride, (uint32_t)p.part_stride * 4u)
                                                  : buffer_over(p.out, 0xfffffffcu);
    const __amdgpu_buffer_rsrc_t r_rs = buffer_over(p.ep != EP_STORE ? p.r : p.out, 0xfffffffcu);
    const uint32_t c_stride = partial ? HW4 : osc4;  // bytes from one output channel to the next
    // channel counts that are multiples of 8 (the usual case) make the bound check uniform: register i exists
    // for both halves of the wavefront or for neither
    const bool whole8 = (CO & 7) == 0;
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        if (o_img[t] < 0) continue;
        const uint32_t o_off = partial ? (uint32_t)((((int64_t)o_img[t] * CO + 4 * kg) * (OH * OW) + o_pix[t]) * 4)
                                       : (uint32_t)(((int64_t)o_img[t] * p.osn + o_pix[t] + (int64_t)(4 * kg) * p.osc) * 4);
        const uint32_t r_off = (uint32_t)(((int64_t)o_img[t] * p.rsn + o_pix[t] + (int64_t)(4 * kg) * p.rsc) * 4);
#pragma unroll
        for (int m = 0; m < MTW; ++m) {
            const int ku0 = co0 + (wm * MTW + m) * 32;  // uniform; register i is channel ku0 + 8*(i/4) + i%4 (+ 4*kg)
            if (!partial && p.ep != EP_STORE) {  // all skip values first: r may alias out
                float rv[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int ku = ku0 + 8 * (i >> 2) + (i & 3);
                    // (a register without a channel re-reads the lane's first one; the value is not used)
                    const bool has = whole8 ? ku < CO : ku + 4 * kg < CO;
                    rv[i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r_rs, has ? r_off : 0u, (uint32_t)(ku < CO ? ku : ku0) * rsc4, 0));
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[m][t][i] = p.ep == EP_ADD ? rv[i] + acc[m][t][i] : rv[i] - acc[m][t][i];
            }
            if (whole8) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int ku = ku0 + 8 * (i >> 2) + (i & 3);
                    if (ku < CO) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[m][t][i]), out_rs, o_off, (uint32_t)ku * c_stride, 0);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int ku = ku0 + 8 * (i >> 2) + (i & 3);
                    if (ku + 4 * kg < CO) __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[m][t][i]), out_rs, o_off, (uint32_t)ku * c_stride, 0);
                }
            }
        }
    }
    // Statistics of what was stored, for the BN layer that reads it next (host: no split, every
    // slot a valid pixel): a channel's 32 * NTW pixels of this wavefront sit in the 32 lanes of one
    // half, NTW per lane; sums about the half's first value, folded 16 channels at a time.
    if constexpr (EMIT) {
#pragma unroll
        for (int m = 0; m < MTW; ++m) {
            float ea[16], eb[16], piv[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int v0 = __float_as_int(acc[m][0][i]);
                const float lo = __int_as_float(__builtin_amdgcn_readlane(v0, 0));
                const float hi = __int_as_float(__builtin_amdgcn_readlane(v0, 32));
                piv[i] = kg ? hi : lo;
                float a = 0.f, b = 0.f;
#pragma unroll
                for (int t = 0; t < NTW; ++t) {
                    const float d = acc[m][t][i] - piv[i];
                    a += d;
                    b += d * d;
                }
                ea[i] = a;
                eb[i] = b;
            }
            fold_16_channels(ea, eb, piv, l32);
            const int i = l32 >> 1;  // the register this lane now holds
            const int ko = co0 + (wm * MTW + m) * 32 + 4 * kg + 8 * (i >> 2) + (i & 3);
            if ((l32 & 1) == 0 && ko < CO) {
                constexpr float inv = 1.f / (32 * NTW);
                const float mean = piv[0] + ea[0] * inv;
                const float m2 = fmaxf(eb[0] - ea[0] * ea[0] * inv, 0.f);
                float2 *dst = reinterpret_cast<float2 *>(p.emit) + (int64_t)ko * p.emit_tiles + (bx * WN + wn);
                *dst = make_float2(mean, m2);
            }
        }
    }
}

}  // namespace c3

}  // namespace

}  // namespace rvn
