// 3x3 convolution (forward and data gradient) with bf16 operands on the CDNA4
// matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation), for the 3x3 units
// c_3(x) = Conv_3x3(ReLU(BN(x))) of Section 2.2 when the block descriptor asks
// for bf16 convolution operands.
//
// GEMM view.  D[ko][pixel] = sum_{tap, c} Wt[ko][tap][c] * A[c][pixel + tap],
// one matrix instruction per (tap, 16 input channels).  Both operands live in
// LDS with the channel innermost (pixel records and (ko, tap) records of KC + 8
// bf16), so every operand read is one 16-byte access per lane.
//
// What this kernel adds to that scheme:
//  * register tiling: a wavefront owns MTW x NTW tiles of 32 x 32 results, so
//    an LDS read feeds NTW (filter) or MTW (activation) matrix instructions;
//  * software pipelining: the global loads of channel chunk i+1 (activations as
//    fp32, filter as prepared bf16) are issued before the matrix instructions
//    of chunk i and are converted and written to LDS after them;
//  * staging by linear quads: an item is 4 consecutive pixels of the band's
//    contiguous range in the image plane, times 8 channels, so the loads are
//    16 bytes whatever the image width; BN scale/shift, ReLU and the bf16
//    rounding happen on the way into LDS;
//  * optional split of the input channels over gridDim.z: partial tiles go to
//    scratch and a second kernel sums them in a fixed order and applies the
//    coupling y = r + conv / reconstruction x = r - conv of Section 3.1
//    (otherwise that is done in the accumulator registers here).
#include <algorithm>

#include "kernels.h"
#include "stats_fold.h"

namespace rvn {

namespace {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef float f4u_t __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kPadK = 8;     // bf16 elements of padding per LDS record
constexpr int kInItems = 2;  // activation staging items per thread and chunk, at most

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
    int TR, IMGS, bands;  // rows and images per pixel block, blocks per image column
    int pix_per_img;      // TR * W
    int n_pix;            // IMGS * TR * W
    int lrows, lcols;     // LDS tile: TR + 2 rows, W + 2 columns
    int q_per_img;        // quads of the widest band range: ceil((TR + 2) * W / 4)
    int in_items;         // IMGS * q_per_img * (KC / 8)
    int chunks, cps;      // channel chunks in total and per split
    float *part;          // partial tiles [split][n][ko][h*w] when gridDim.z > 1
    int64_t part_stride;
    // EMIT instances (no split, every pixel slot of every workgroup a valid pixel): per channel and
    // wavefront the mean and centred sum of squares of the 32 * NTW pixels it stores, at
    // emit[(channel * emit_tiles + blockIdx.x * WN + wn) * 2]
    float *emit;
    int emit_tiles;
};

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
template <int WM, int MTW, int NTW, int KC, bool EMIT = false, int NI = kInItems>
__global__ __launch_bounds__(kThreads, 2) void conv3x3_bf16_k(const C3Args p) {
    constexpr int WN = 4 / WM;
    constexpr int REC = KC + kPadK, OCTS = KC / 8;
    constexpr int CH = WM * MTW * 32;  // output channels per workgroup
    constexpr int W_ITEMS = CH * 9 * OCTS, W_PER = (W_ITEMS + kThreads - 1) / kThreads;
    extern __shared__ __align__(16) uint16_t smem16[];
    uint16_t *in_lds = smem16;                                    // [IMGS][lrows][lcols][REC]
    uint16_t *w_lds = smem16 + p.IMGS * p.lrows * p.lcols * REC;  // [CH][9][REC]
    float *ss_lds = reinterpret_cast<float *>(w_lds + CH * 9 * REC);  // [2][CI]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int band = blockIdx.x % p.bands, img_grp = blockIdx.x / p.bands;
    const int n0 = img_grp * p.IMGS, row0 = band * p.TR;
    const int co0 = blockIdx.y * CH;
    const int N = p.N, H = p.H, W = p.W, CI = p.CI, CO = p.CO;
    const int l32 = lane & 31, kg = lane >> 5;
    const bool bn = p.scale_shift != nullptr;

    // ---- zero the activation tile once (halo, rows outside the image, unused
    //      slots stay zero) and fetch scale/shift
    {
        const int n16 = p.IMGS * p.lrows * p.lcols * REC / 8;
        for (int e = tid; e < n16; e += kThreads) reinterpret_cast<uint4_t *>(in_lds)[e] = uint4_t{0u, 0u, 0u, 0u};
        if (bn)
            for (int e = tid; e < 2 * CI; e += kThreads) ss_lds[e] = p.scale_shift[e];
    }

    // ---- this thread's activation items: (image, quad of the band's pixel range, channel octet)
    const int start_row = max(0, row0 - 1), end_row = min(H, row0 + p.TR + 1);
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
        it_off[i] = live ? (uint32_t)(((int64_t)n * p.isn + start_row * W + ld) * 4) : 0u;
        it_rec[i] = (img * p.lrows + (row - (row0 - 1))) * p.lcols + 1 + col;
        const int nvalid = live ? 4 : 0;
        it_info[i] = col | (nvalid << 16) | (oc << 24);
    }

    // ---- this lane's pixel in each of its NTW pixel groups
    int b_rec[NTW], o_img[NTW], o_pix[NTW];
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        const int f = (wn * NTW + t) * 32 + l32;
        const int img = f / p.pix_per_img, rem = f - img * p.pix_per_img;
        const int rr = rem / W, cc = rem - rr * W;
        const bool ok = f < p.n_pix && n0 + img < N && row0 + rr < H;
        b_rec[t] = f < p.n_pix ? (img * p.lrows + rr) * p.lcols + cc : 0;
        o_img[t] = ok ? n0 + img : -1;
        o_pix[t] = (row0 + rr) * W + cc;
    }

    float16_t acc[MTW][NTW];
#pragma unroll
    for (int m = 0; m < MTW; ++m)
#pragma unroll
        for (int t = 0; t < NTW; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][t][i] = 0.f;

    constexpr int SETS = NI == 1 ? 2 : 1;  // register sets of activation loads
    f4u_t gin[SETS][NI][8];
    uint4_t gw[W_PER];
    const char *const in_base = reinterpret_cast<const char *>(p.in);
    const int64_t isc_b = p.isc * 4;

    // global -> registers: the activations of chunk c0 into register set `set`, the filter of chunk c0
    auto g2r_act = [&](f4u_t (&g)[NI][8], int c0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int oc = it_info[i] >> 24;
            // octets past the last channel read the chunk's first octet instead and are zeroed later
            const uint32_t off = it_off[i] + (c0 + oc * 8 < CI ? (uint32_t)(oc * 8 * isc_b) : 0u);
#pragma unroll
            for (int k = 0; k < 8; ++k)
                g[i][k] = *reinterpret_cast<const f4u_t *>(in_base + (int64_t)(c0 + k) * isc_b + off);
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
    auto r2l_act = [&](const f4u_t (&g)[NI][8], int c0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int info = it_info[i];
            const int col = info & 0xffff, nvalid = (info >> 16) & 15, oc = info >> 24;
            if (nvalid == 0) continue;
            const bool chan_ok = c0 + oc * 8 < CI;
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

    const int chunk0 = blockIdx.z * p.cps, chunk1 = min(p.chunks, chunk0 + p.cps);
    g2r_w(chunk0 * KC);
    g2r_act(gin[0], chunk0 * KC);
    if (SETS == 2 && chunk0 + 1 < chunk1) g2r_act(gin[SETS - 1], (chunk0 + 1) * KC);
    __syncthreads();  // tile zeroed, scale/shift in LDS
    r2l_w();
    r2l_act(gin[0], chunk0 * KC);
    __syncthreads();
    if constexpr (SETS == 1) {
        for (int ch = chunk0; ch < chunk1; ++ch) {
            if (ch + 1 < chunk1) {
                g2r_w((ch + 1) * KC);
                g2r_act(gin[0], (ch + 1) * KC);
            }
            multiply();
            if (ch + 1 < chunk1) {
                __syncthreads();  // every wavefront has read chunk ch
                r2l_w();
                r2l_act(gin[0], (ch + 1) * KC);
                __syncthreads();
            }
        }
    } else {
        // LDS holds chunk ch; set 1 holds chunk ch + 1 (in flight), set 0 is free -- and the other way
        // round one chunk later.  The filter (small, cached) keeps one chunk of lookahead and is requested
        // before the activations two chunks ahead, so that waiting for it does not wait for them.
        for (int ch = chunk0; ch < chunk1; ch += 2) {
            if (ch + 1 < chunk1) g2r_w((ch + 1) * KC);
            if (ch + 2 < chunk1) g2r_act(gin[0], (ch + 2) * KC);
            multiply();
            if (ch + 1 >= chunk1) break;
            __syncthreads();  // every wavefront has read chunk ch
            r2l_w();
            r2l_act(gin[SETS - 1], (ch + 1) * KC);
            __syncthreads();
            if (ch + 2 < chunk1) g2r_w((ch + 2) * KC);
            if (ch + 3 < chunk1) g2r_act(gin[SETS - 1], (ch + 3) * KC);
            multiply();
            if (ch + 2 < chunk1) {
                __syncthreads();
                r2l_w();
                r2l_act(gin[0], (ch + 2) * KC);
                __syncthreads();
            }
        }
    }

    // ---- epilogue: register i of a lane is channel 8*(i/4) + 4*kg + i%4 of its pixel.
    //      Every access is a buffer access: a 32-bit per-lane byte offset (image, pixel, 4*kg channels)
    //      plus a wavefront-uniform byte offset (the channel without the lane's 4*kg) that lives in scalar
    //      registers; the host keeps every tensor handed to one launch below 4 GB.  With a 64-bit address
    //      per lane and access, address arithmetic was half of the kernel's vector instructions.
    const bool partial = gridDim.z > 1;
    const uint32_t HW4 = (uint32_t)(H * W) * 4u;
    const uint32_t osc4 = (uint32_t)p.osc * 4u, rsc4 = (uint32_t)p.rsc * 4u;
    const __amdgpu_buffer_rsrc_t out_rs = partial ? buffer_over(p.part + blockIdx.z * p.part_stride, (uint32_t)p.part_stride * 4u)
                                                  : buffer_over(p.out, 0xfffffffcu);
    const __amdgpu_buffer_rsrc_t r_rs = buffer_over(p.ep != EP_STORE ? p.r : p.out, 0xfffffffcu);
    const uint32_t c_stride = partial ? HW4 : osc4;  // bytes from one output channel to the next
    // channel counts that are multiples of 8 (the usual case) make the bound check uniform: register i exists
    // for both halves of the wavefront or for neither
    const bool whole8 = (CO & 7) == 0;
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        if (o_img[t] < 0) continue;
        const uint32_t o_off = partial ? (uint32_t)((((int64_t)o_img[t] * CO + 4 * kg) * (H * W) + o_pix[t]) * 4)
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
                float2 *dst = reinterpret_cast<float2 *>(p.emit) + (int64_t)ko * p.emit_tiles + ((int)blockIdx.x * WN + wn);
                *dst = make_float2(mean, m2);
            }
        }
    }
}

// out = ep(r, sum_s part[s]) over dense partial tiles [S][n][c][hw], summed in
// the order s = 0, 1, ...  EMIT (host: h*w a multiple of 64, total a multiple of
// the workgroup size, so a wavefront holds 64 consecutive pixels of one plane):
// the wavefront also leaves the mean and centred sum of squares of what it
// stores at emit[(c * emit_tiles + n * (h*w / 64) + pixel / 64) * 2], for the
// BN layer that reads the tensor next.
template <bool EMIT>
__global__ __launch_bounds__(kThreads) void splitk_reduce_k(const float *__restrict__ part, int64_t part_stride, int S,
                                                            int C, int HW, int64_t total, const float *r,
                                                            int64_t rsn, int64_t rsc, float *out, int64_t osn,
                                                            int64_t osc, int ep, float *emit, int emit_tiles) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    float v = part[i];
    for (int s = 1; s < S; ++s) v += part[(int64_t)s * part_stride + i];
    const int64_t plane = i / HW;
    const int pix = (int)(i - plane * HW);
    const int64_t n = plane / C;
    const int c = (int)(plane - n * C);
    if (ep != EP_STORE) {
        const float rv = r[n * rsn + (int64_t)c * rsc + pix];
        v = ep == EP_ADD ? rv + v : rv - v;
    }
    out[n * osn + (int64_t)c * osc + pix] = v;
    if constexpr (EMIT) {
        const float pivot = __shfl(v, 0, 64);
        float a = v - pivot, b = a * a;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            a += __shfl_xor(a, off, 64);
            b += __shfl_xor(b, off, 64);
        }
        if ((threadIdx.x & 63) == 0) {
            const float mean = pivot + a * (1.f / 64.f);
            const float m2 = fmaxf(b - a * a * (1.f / 64.f), 0.f);
            const int tile = (int)n * (HW >> 6) + (pix >> 6);
            reinterpret_cast<float2 *>(emit)[(int64_t)c * emit_tiles + tile] = make_float2(mean, m2);
        }
    }
}

struct C3Plan {
    int WM, MTW, NTW, KC, TR, IMGS, bands, lrows, lcols, q_per_img, in_items, chunks, S, cps;
    size_t lds_bytes;
    bool ok;
};

C3Plan plan_c3(int ci, int co, const Geo &g) {
    C3Plan pl{};
    pl.ok = false;
    if (ci % 8 != 0 || g.w < 4 || ci > 4096) return pl;
    // Output channels per workgroup and the wavefront arrangement.
    // 64 output channels per workgroup at most, the four wavefronts side by side along the pixels: with
    // 128 channels (two wavefronts stacked) the wide layers were 5-10 % slower (twice the filter tile per
    // workgroup, half as many pixel slots).
    pl.WM = 1; pl.MTW = co <= 32 ? 1 : 2; pl.NTW = 2;
    const int ch = pl.WM * pl.MTW * 32, slots = (4 / pl.WM) * pl.NTW * 32;
    // One chunk of 32 channels when that is the whole input; otherwise chunks of
    // 16, which pipeline better (measured on 64-, 56- and 32-channel layers).
    pl.KC = ci == 32 && ch <= 64 ? 32 : 16;
    const int rec = pl.KC + kPadK, octs = pl.KC / 8;
    // Pixel block: the fullest block of whole rows (or whole images) that fits.
    double best = -1.0;
    for (int imgs = 1; imgs <= 16 && imgs <= g.n; ++imgs) {
        for (int tr = imgs > 1 ? g.h : 1; tr <= g.h; ++tr) {
            const int npix = imgs * tr * g.w;
            if (npix > slots) break;
            const int lrows = tr + 2, lcols = g.w + 2;
            const int q = ((tr + 2) * g.w + 3) / 4;
            const int items = imgs * q * octs;
            const size_t bytes = ((size_t)imgs * lrows * lcols + (size_t)ch * 9) * rec * 2 + (size_t)ci * 8;
            if (items > kInItems * kThreads || bytes > 76 * 1024) break;
            const int bands = (g.h + tr - 1) / tr, groups = (g.n + imgs - 1) / imgs;
            const double useful = (double)g.n * g.h * g.w, issued = (double)groups * bands * slots;
            const double score = useful / issued;
            if (score > best) {
                best = score;
                pl.TR = tr; pl.IMGS = imgs; pl.bands = bands; pl.lrows = lrows; pl.lcols = lcols;
                pl.q_per_img = q; pl.in_items = items; pl.lds_bytes = bytes;
                pl.ok = true;
            }
        }
    }
    if (!pl.ok) return pl;
    pl.chunks = (ci + pl.KC - 1) / pl.KC;
    const int64_t wgs = (int64_t)((g.n + pl.IMGS - 1) / pl.IMGS) * pl.bands * ((co + ch - 1) / ch);
    pl.S = 1;
    // Too few workgroups for the chip (measured: at most one per two compute
    // units): split the input channels over gridDim.z as well.
    if (wgs <= 128 && pl.chunks >= 4) pl.S = (int)std::min<int64_t>(pl.chunks / 2, (512 + wgs - 1) / wgs);
    pl.cps = (pl.chunks + pl.S - 1) / pl.S;
    pl.S = (pl.chunks + pl.cps - 1) / pl.cps;
    return pl;
}

template <int WM, int MTW, int NTW, int KC, bool EMIT, int NI>
void launch_c3_items(Ctx &cx, const C3Plan &pl, const C3Args &a, dim3 grid) {
    static bool raised = false;  // more than 64 KB of dynamic LDS has to be asked for once
    if (!raised && !cx.dry) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(conv3x3_bf16_k<WM, MTW, NTW, KC, EMIT, NI>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        if (e != hipSuccess) {
            cx.fail(e);
            return;
        }
        raised = true;
    }
    cx.run(conv3x3_bf16_k<WM, MTW, NTW, KC, EMIT, NI>, grid, dim3(kThreads), pl.lds_bytes, a);
}

template <int WM, int MTW, int NTW, int KC, bool EMIT>
void launch_c3_variant(Ctx &cx, const C3Plan &pl, const C3Args &a, dim3 grid) {
    // one staging item per thread at most: the variant whose activation loads run two chunks ahead
    if (pl.in_items <= kThreads) launch_c3_items<WM, MTW, NTW, KC, EMIT, 1>(cx, pl, a, grid);
    else launch_c3_items<WM, MTW, NTW, KC, EMIT, kInItems>(cx, pl, a, grid);
}

template <int WM, int MTW, int NTW, int KC>
void launch_c3(Ctx &cx, const C3Plan &pl, const C3Args &a, dim3 grid) {
    if (a.emit) launch_c3_variant<WM, MTW, NTW, KC, true>(cx, pl, a, grid);
    else launch_c3_variant<WM, MTW, NTW, KC, false>(cx, pl, a, grid);
}

}  // namespace

bool conv3x3_bf16_ok(int ci, int co, const Geo &g) { return plan_c3(ci, co, g).ok; }

size_t conv3x3_bf16_scratch_floats(int ci, int co, const Geo &g) {
    const C3Plan pl = plan_c3(ci, co, g);
    return pl.ok && pl.S > 1 ? (size_t)pl.S * g.n * co * g.h * g.w : 0;
}

bool conv3x3_bf16(Ctx &cx, View in, const float *scale_shift, const uint16_t *wq, int ci, int co, Geo g,
                  Epilogue ep, const View *r, View out, float *scratch) {
    if (!wq) return false;
    const C3Plan pl = plan_c3(ci, co, g);
    if (!pl.ok || (pl.S > 1 && !scratch)) return false;
    // lane offsets into `in`, `out`, `r` and the partial tiles are 32-bit byte offsets
    const int64_t lim = (int64_t)1 << 32;
    if (((int64_t)g.n * in.sn + (int64_t)ci * in.sc) * 4 >= lim || ((int64_t)g.n * out.sn + (int64_t)co * out.sc) * 4 >= lim ||
        (r && ((int64_t)g.n * r->sn + (int64_t)co * r->sc) * 4 >= lim) || (int64_t)g.n * co * g.h * g.w * 4 >= lim)
        return false;
    C3Args a{};
    a.in = in.p; a.isn = in.sn; a.isc = in.sc;
    a.scale_shift = scale_shift;
    a.wq = wq; a.CIP = (ci + 7) / 8 * 8;
    a.r = r ? r->p : nullptr; a.rsn = r ? r->sn : 0; a.rsc = r ? r->sc : 0;
    a.out = out.p; a.osn = out.sn; a.osc = out.sc;
    a.N = g.n; a.H = g.h; a.W = g.w; a.CI = ci; a.CO = co; a.ep = (int)ep;
    a.TR = pl.TR; a.IMGS = pl.IMGS; a.bands = pl.bands;
    a.pix_per_img = pl.TR * g.w; a.n_pix = pl.IMGS * pl.TR * g.w;
    a.lrows = pl.lrows; a.lcols = pl.lcols; a.q_per_img = pl.q_per_img; a.in_items = pl.in_items;
    a.chunks = pl.chunks; a.cps = pl.cps;
    a.part = scratch; a.part_stride = (int64_t)g.n * co * g.h * g.w;
    const int ch = pl.WM * pl.MTW * 32;
    const dim3 grid((unsigned)(pl.bands * ((g.n + pl.IMGS - 1) / pl.IMGS)), (unsigned)((co + ch - 1) / ch), (unsigned)pl.S);
    // Statistics of the output for the BN layer that reads it next: no split (for split launches see
    // below), and every pixel slot of every workgroup a valid pixel (whole blocks of rows or images).
    const int wn_count = 4 / pl.WM, slots = wn_count * 2 * 32, tiles = (int)grid.x * wn_count;
    const bool whole = a.n_pix == slots && g.n % pl.IMGS == 0 && g.h % pl.TR == 0;
    if (cx.want_emit && cx.emit_buf && pl.S == 1 && whole && (size_t)co * tiles * 2 <= cx.emit_floats) {
        a.emit = cx.emit_buf;
        a.emit_tiles = tiles;
        cx.emitted = EmittedStats{out.p, out.sn, out.sc, co, g.n, g.h, g.w, tiles, 64};
    }
    bool launched = true;
    if (pl.WM == 1 && pl.MTW == 1 && pl.KC == 16) launch_c3<1, 1, 2, 16>(cx, pl, a, grid);
    else if (pl.WM == 1 && pl.MTW == 1 && pl.KC == 32) launch_c3<1, 1, 2, 32>(cx, pl, a, grid);
    else if (pl.WM == 1 && pl.MTW == 2 && pl.KC == 16) launch_c3<1, 2, 2, 16>(cx, pl, a, grid);
    else if (pl.WM == 1 && pl.MTW == 2 && pl.KC == 32) launch_c3<1, 2, 2, 32>(cx, pl, a, grid);
    else launched = false;
    if (!launched) {
        cx.emitted = EmittedStats{};
        return false;
    }
    if (pl.S > 1) {
        const int64_t total = a.part_stride;
        // the values are final only here: this kernel leaves the statistics when its wavefronts are whole
        // runs of 64 pixels of one plane
        const int hw = g.h * g.w, rtiles = g.n * (hw / 64);
        const dim3 rgrid((unsigned)((total + kThreads - 1) / kThreads));
        // (a launch of its own in the accounts; the convolution's algorithmic bytes were counted with the first)
        const bool go = cx.launch(K_SPLITK_REDUCE, 0.0);
        if (cx.want_emit && cx.emit_buf && hw % 64 == 0 && total % kThreads == 0 &&
            (size_t)co * rtiles * 2 <= cx.emit_floats) {
            cx.emitted = EmittedStats{out.p, out.sn, out.sc, co, g.n, g.h, g.w, rtiles, 64};
            if (go)
                cx.run(splitk_reduce_k<true>, rgrid, dim3(kThreads), 0, scratch, a.part_stride, pl.S, co, hw, total, a.r,
                       a.rsn, a.rsc, a.out, a.osn, a.osc, a.ep, cx.emit_buf, rtiles);
        } else if (go) {
            cx.run(splitk_reduce_k<false>, rgrid, dim3(kThreads), 0, scratch, a.part_stride, pl.S, co, hw, total, a.r,
                   a.rsn, a.rsc, a.out, a.osn, a.osc, a.ep, (float *)nullptr, 0);
        }
    }
    return true;
}

}  // namespace rvn
