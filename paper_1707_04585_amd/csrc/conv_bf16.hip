// Implicit-GEMM convolution (forward and data gradient) with bf16 operands on
// the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation), for the
// units c_k(x) = Conv_kxk(ReLU(BN(x))) of Section 2.2 when the block descriptor
// asks for bf16 convolution operands.
//
// GEMM view.  D[ko][pixel] = sum_K Wt[ko][K] * A[K][pixel], K = (tap, c) with
// the input channel c running fastest.  One matrix instruction multiplies a
// 32(ko) x 16(K) filter slice by a 16(K) x 32(pixel) activation slice: 16
// consecutive input channels at one filter tap.  Each lane feeds 8 consecutive
// K values of its row/column, i.e. 8 consecutive channels of one pixel, so both
// operands live in LDS with the channel innermost ([pixel][channel] and
// [ko][tap][channel], bf16) and are read with single 16-byte accesses.
//
// Staging.  The input is fp32 NCHW in HBM.  A thread loads, for 4 consecutive
// pixels of a row, 8 consecutive channels (8 coalesced 16-byte loads), applies
// the BN scale/shift and ReLU of the unit (forward) or nothing (data gradient),
// rounds to bf16 (nearest even) and writes four 16-byte pixel records; halo
// rows/columns and padded channels are zero.  Filters are gathered from their
// fp32 [cout][cin][k][k] layout (transposed and flipped for the data gradient)
// into K order.  Output channels sit on the M side: a lane's 16 results are 16
// channels of one pixel, 32 lanes hold 32 consecutive pixels, so results go to
// NCHW memory in 128-byte runs and the coupling y = r + acc / reconstruction
// x = r - acc of Section 3.1 is applied in the accumulator registers.
//
// Work decomposition.  A workgroup (4 wavefronts) owns a block of pixels (TR
// full rows of IMGS images, at most 4*NT*32 pixels) and MT*32 output channels;
// wavefront w takes the pixel groups w*NT .. w*NT+NT-1.  Input channels are
// consumed KC at a time.
#include <algorithm>

#include "kernels.h"
#include "prep_filter.h"

namespace rvn {

namespace {

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kPadK = 8;  // bf16 elements of padding per LDS record (spreads 16-byte reads over the banks)

struct Bf16Args {
    const float *in;  // x (forward) or upstream gradient (data gradient), fp32 NCHW
    int64_t isn, isc;
    const float *scale_shift;  // [2*CI]: a = max(in*scale + shift, 0); null = use `in` as is
    const float *w;            // [CO][CI][KS][KS] forward; [CI][CO][KS][KS] read transposed+flipped otherwise
    const uint16_t *wq;        // or null: the same filter already in bf16 and K order, [CO][KS*KS][CIP]
    int CIP;                   // channel pitch of wq (a multiple of 8)
    const float *r;            // skip operand of the epilogue (may alias out)
    int64_t rsn, rsc;
    float *out;
    int64_t osn, osc;
    int N, H, W, CI, CO;
    int ep, transposed;
    int TR, IMGS, bands;  // rows and images per pixel block, blocks per image column
    int pix_per_img;      // TR * W
    int n_pix;            // IMGS * TR * W (<= 4 * NT * 32)
    int lrows, lcols;     // LDS tile: TR + KS - 1 rows, W + KS - 1 columns
    int Wq;               // 4-pixel groups per image row
    int in_items;         // staging items of the input tile: IMGS * lrows * Wq * (KC / 8)
};

__device__ __forceinline__ uint32_t bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
// Two floats to a pair of bf16 (nearest even): one v_cvt_pk_bf16_f32.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    const float2_t v = {lo, hi};
    const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<const uint32_t *>(&b);
}

template <int KS, int MT, int NT, int KC>
__global__ __launch_bounds__(kThreads) void conv_bf16_k(const Bf16Args p) {
    constexpr int KS2 = KS * KS, PAD = KS / 2;
    constexpr int REC = KC + kPadK;    // bf16 elements per pixel record / per (ko, tap) filter record
    constexpr int CH = MT * 32;        // output channels per workgroup
    constexpr int W_ITEMS = CH * KS2 * (KC / 8);
    extern __shared__ __align__(16) uint16_t smem16[];
    uint16_t *in_lds = smem16;                                    // [IMGS][lrows][lcols][REC]
    uint16_t *w_lds = smem16 + p.IMGS * p.lrows * p.lcols * REC;  // [CH][KS2][REC]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int band = blockIdx.x % p.bands, img_grp = blockIdx.x / p.bands;
    const int n0 = img_grp * p.IMGS, row0 = band * p.TR;
    const int co0 = blockIdx.y * CH;
    const int N = p.N, H = p.H, W = p.W, CI = p.CI, CO = p.CO;
    const int l32 = lane & 31, kg = lane >> 5;  // pixel / ko within a 32-group; which 8 of the 16 K values

    // This lane's pixel in each of its NT pixel groups: LDS record index of the
    // pixel at tap (0, 0), and where its results go.
    int b_rec[NT], o_img[NT], o_pix[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int f = (wave * NT + t) * 32 + l32;
        const int img = f / p.pix_per_img, rem = f - img * p.pix_per_img;
        const int rr = rem / W, cc = rem - rr * W;
        const bool ok = f < p.n_pix && n0 + img < N && row0 + rr < H;
        b_rec[t] = f < p.n_pix ? (img * p.lrows + rr) * p.lcols + cc : 0;
        o_img[t] = ok ? n0 + img : -1;
        o_pix[t] = (row0 + rr) * W + cc;
    }

    float16_t acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][t][i] = 0.f;

    const bool vec = (W & 3) == 0 && (p.isn & 3) == 0 && (p.isc & 3) == 0 && (reinterpret_cast<uintptr_t>(p.in) & 15) == 0;
    const int octs = KC / 8;

    for (int c0 = 0; c0 < CI; c0 += KC) {
        __syncthreads();  // previous chunk fully consumed
        // ---- input tile: item = (image, tile row, 4-pixel group, channel octet)
        for (int e = tid; e < p.in_items; e += kThreads) {
            const int oc = e % octs;
            int t = e / octs;
            const int qx = t % p.Wq;
            t /= p.Wq;
            const int lr = t % p.lrows, img = t / p.lrows;
            const int n = n0 + img, row = row0 - PAD + lr, col = qx * 4, chb = c0 + oc * 8;
            const bool live = n < N && row >= 0 && row < H;
            float v[8][4];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                v[k][0] = v[k][1] = v[k][2] = v[k][3] = 0.f;
                if (live && chb + k < CI) {
                    const float *src = p.in + (int64_t)n * p.isn + (int64_t)(chb + k) * p.isc + row * W + col;
                    if (vec) {
                        const float4 q = *reinterpret_cast<const float4 *>(src);
                        v[k][0] = q.x; v[k][1] = q.y; v[k][2] = q.z; v[k][3] = q.w;
                    } else {
                        v[k][0] = src[0];
                        if (col + 1 < W) v[k][1] = src[1];
                        if (col + 2 < W) v[k][2] = src[2];
                        if (col + 3 < W) v[k][3] = src[3];
                    }
                    if (p.scale_shift) {
                        const float sc = p.scale_shift[chb + k], sh = p.scale_shift[CI + chb + k];
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[k][j] = fmaxf(fmaf(v[k][j], sc, sh), 0.f);
                    }
                }
            }
            uint16_t *dst = in_lds + ((img * p.lrows + lr) * p.lcols + PAD + col) * REC + oc * 8;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (col + j >= W) break;
                uint4 rec;
                rec.x = pack2(v[0][j], v[1][j]);
                rec.y = pack2(v[2][j], v[3][j]);
                rec.z = pack2(v[4][j], v[5][j]);
                rec.w = pack2(v[6][j], v[7][j]);
                *reinterpret_cast<uint4 *>(dst + j * REC) = rec;
            }
        }
        if (KS == 3) {  // zero halo columns: records (row, 0) and (row, lcols - 1)
            const int n_rows = p.IMGS * p.lrows;
            for (int e = tid; e < n_rows * 2 * octs; e += kThreads) {
                const int oc = e % octs, side = (e / octs) & 1, rw = e / (2 * octs);
                uint16_t *dst = in_lds + (rw * p.lcols + (side ? p.lcols - 1 : 0)) * REC + oc * 8;
                *reinterpret_cast<uint4 *>(dst) = make_uint4(0u, 0u, 0u, 0u);
            }
        }
        // ---- filter tile: item = (ko, tap, channel octet) -> 8 K-consecutive values
        if (p.wq) {
            for (int e = tid; e < W_ITEMS; e += kThreads) {
                const int oc = e % octs;
                const int t = e / octs;  // = kol * KS2 + tap
                const int ko = co0 + t / KS2, chb = c0 + oc * 8;
                uint4 rec = make_uint4(0u, 0u, 0u, 0u);
                if (ko < CO && chb < p.CIP)
                    rec = *reinterpret_cast<const uint4 *>(p.wq + ((int64_t)co0 * KS2 + t) * p.CIP + chb);
                *reinterpret_cast<uint4 *>(w_lds + t * REC + oc * 8) = rec;
            }
        } else {
            for (int e = tid; e < W_ITEMS; e += kThreads) {
                const int oc = e % octs;
                int t = e / octs;
                const int tap = t % KS2, kol = t / KS2;
                const int ko = co0 + kol, chb = c0 + oc * 8;
                float v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    v[k] = 0.f;
                    const int ch = chb + k;
                    if (ko < CO && ch < CI)
                        v[k] = p.transposed ? p.w[((int64_t)ch * CO + ko) * KS2 + (KS2 - 1 - tap)]
                                            : p.w[((int64_t)ko * CI + ch) * KS2 + tap];
                }
                uint4 rec;
                rec.x = pack2(v[0], v[1]);
                rec.y = pack2(v[2], v[3]);
                rec.z = pack2(v[4], v[5]);
                rec.w = pack2(v[6], v[7]);
                *reinterpret_cast<uint4 *>(w_lds + (kol * KS2 + tap) * REC + oc * 8) = rec;
            }
        }
        __syncthreads();
        // ---- multiply
#pragma unroll
        for (int rr = 0; rr < KS; ++rr) {
#pragma unroll
            for (int ss = 0; ss < KS; ++ss) {
#pragma unroll
                for (int ks = 0; ks < KC / 16; ++ks) {
                    bf16x8_t a[MT];
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        a[m] = *reinterpret_cast<const bf16x8_t *>(
                            w_lds + ((m * 32 + l32) * KS2 + rr * KS + ss) * REC + ks * 16 + kg * 8);
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const bf16x8_t b = *reinterpret_cast<const bf16x8_t *>(
                            in_lds + (b_rec[t] + rr * p.lcols + ss) * REC + ks * 16 + kg * 8);
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            acc[m][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m], b, acc[m][t], 0, 0, 0);
                    }
                }
            }
        }
    }

    // ---- epilogue: register i of a lane is channel 8*(i/4) + 4*kg + i%4 of its pixel
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (o_img[t] < 0) continue;
        float *const dst = p.out + (int64_t)o_img[t] * p.osn + o_pix[t];
        const float *const rsrc = p.ep != EP_STORE ? p.r + (int64_t)o_img[t] * p.rsn + o_pix[t] : nullptr;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int ko = co0 + m * 32 + 8 * (i >> 2) + 4 * kg + (i & 3);
                if (ko >= CO) continue;
                float v = acc[m][t][i];
                if (p.ep != EP_STORE) {
                    const float rv = rsrc[(int64_t)ko * p.rsc];
                    v = p.ep == EP_ADD ? rv + v : rv - v;
                }
                dst[(int64_t)ko * p.osc] = v;
            }
        }
    }
}

struct Bf16Plan {
    int MT, NT, KC, TR, IMGS, bands, lrows, lcols, Wq, in_items;
    size_t lds_bytes;
    bool ok;
};

// Pixel block (TR rows of IMGS images), pixel groups per wavefront and channel
// chunk: the fullest matrix-instruction columns that fit 64 KB of LDS.
Bf16Plan plan_bf16(int ci, int co, int ks, const Geo &g) {
    Bf16Plan best{};
    best.ok = false;
    double best_score = -1.0;
    // Channels per chunk: as many as the problem has, up to 128 (1x1) / 64 (3x3),
    // if the tiles still fit; fewer, larger chunks mean fewer barriers per result.
    for (int kc : {16, 32, 64, 128}) {
    if (kc > 16 && kc / 2 >= ci) continue;
    if (ks == 3 && kc > 64) continue;
    const int rec = kc + kPadK;
    for (int mt : {1, 2, 4}) {
        if (mt > 1 && co <= (mt / 2) * 32) continue;
        const int groups_y = (co + mt * 32 - 1) / (mt * 32);
        for (int nt : {1, 2, 4}) {
            if (mt * nt > 4) continue;  // 64 accumulator registers at most: three workgroups per compute unit
            const int slots = kWaves * nt * 32;
            for (int imgs = 1; imgs <= 16 && imgs <= g.n; ++imgs) {
                for (int tr = imgs > 1 ? g.h : 1; tr <= g.h; ++tr) {
                    const int npix = imgs * tr * g.w;
                    if (npix > slots) break;
                    const int lrows = tr + ks - 1, lcols = g.w + ks - 1;
                    const size_t bytes = ((size_t)imgs * lrows * lcols + (size_t)mt * 32 * ks * ks) * rec * 2;
                    if (bytes > 64 * 1024) break;
                    const int bands = (g.h + tr - 1) / tr, groups = (g.n + imgs - 1) / imgs;
                    // useful results over issued matrix-instruction results, whole problem
                    const double useful = (double)g.n * g.h * g.w * co;
                    const double issued = (double)groups * bands * slots * groups_y * mt * 32;
                    double score = useful / issued;
                    // first enough workgroups to give every compute unit two; then
                    // larger tiles, which re-read input and filter tiles less often
                    const double wgs = (double)groups * bands * groups_y;
                    if (wgs < 512) score *= 0.25 + 0.75 * wgs / 512;
                    score *= 1.0 + 0.03 * nt + 0.03 * mt + (kc >= 128 ? 0.09 : kc >= 64 ? 0.06 : kc >= 32 ? 0.03 : 0.0);
                    if (score > best_score) {
                        best_score = score;
                        best.MT = mt; best.NT = nt; best.KC = kc; best.TR = tr; best.IMGS = imgs; best.bands = bands;
                        best.lrows = lrows; best.lcols = lcols; best.Wq = (g.w + 3) / 4;
                        best.in_items = imgs * lrows * best.Wq * (kc / 8);
                        best.lds_bytes = bytes;
                        best.ok = true;
                    }
                }
            }
        }
    }
    }
    return best;
}

__global__ __launch_bounds__(kThreads) void prep_filter_k(const PrepArgs p) { prep_filter_body(p, blockIdx.x); }

}  // namespace

size_t conv_bf16_scratch_floats(int ci, int co, int ks, const Geo &g) {
    return ks == 3 ? conv3x3_bf16_scratch_floats(ci, co, g) : 0;
}

size_t filter_bf16_elems(int rows, int cols_k, int ks) {
    const size_t n = (size_t)rows * ks * ks * ((cols_k + 7) / 8 * 8);
    return ks == 1 ? std::max(n, filter_1x1_elems(rows, cols_k)) : n;
}

PrepArgs plan_filter_prep(const FilterPrep *f, int count, Geo g, double *bytes_out) {
    PrepArgs a{};
    int blocks = 0;
    double bytes = 0.0;
    auto add = [&](const FilterPrep &fp, uint16_t *q, int kind, int kp, int64_t n) {
        PrepJob &jb = a.job[a.jobs++];
        jb.w = fp.w; jb.q = q; jb.CO = fp.cout; jb.CI = fp.cin; jb.KS2 = fp.ks * fp.ks; jb.kind = kind; jb.KP = kp;
        jb.block0 = blocks; jb.n = n;
        blocks += (int)((n + kThreads - 1) / kThreads);
        bytes += 2.0 * n * (kind <= 1 ? jb.KS2 : 1);
    };
    for (int i = 0; i < count && i < 3; ++i) {
        const FilterPrep &fp = f[i];
        if (!fp.qf && !fp.qb) continue;
        bytes += 4.0 * fp.cin * fp.cout * fp.ks * fp.ks;
        const int cip = (fp.cin + 7) / 8 * 8, cop = (fp.cout + 7) / 8 * 8, ks2 = fp.ks * fp.ks;
        if (fp.qf) {
            if (fp.ks == 1 && conv1x1_direct_ok(fp.cin, g))
                add(fp, fp.qf, 2, (fp.cin + 15) / 16, (int64_t)filter_1x1_elems(fp.cout, fp.cin));
            else
                add(fp, fp.qf, 0, cip, (int64_t)fp.cout * cip);
        }
        if (fp.qb) {
            if (fp.ks == 1 && conv1x1_direct_ok(fp.cout, g))
                add(fp, fp.qb, 3, (fp.cout + 15) / 16, (int64_t)filter_1x1_elems(fp.cin, fp.cout));
            else
                add(fp, fp.qb, 1, cop, (int64_t)fp.cin * cop);
        }
    }
    a.blocks = blocks;
    if (bytes_out) *bytes_out = bytes;
    return a;
}

void prep_filters_bf16(Ctx &cx, const PrepArgs &a, double bytes) {
    if (a.jobs == 0) return;
    if (!cx.launch(K_PREP_FILTER, bytes)) return;
    cx.run(prep_filter_k, dim3((unsigned)a.blocks), dim3(kThreads), 0, a);
}

bool conv_bf16(Ctx &cx, View in, const float *scale_shift, const float *w, const uint16_t *wq, bool transposed,
               int ci, int co, int ks, Geo g, Epilogue ep, const View *r, View out, float *scratch) {
    if (ks == 1 && wq && conv1x1_direct_ok(ci, g)) return conv1x1_bf16(cx, in, scale_shift, wq, ci, co, g, ep, r, out);
    if (ks == 3 && wq && conv3x3_bf16(cx, in, scale_shift, wq, ci, co, g, ep, r, out, scratch)) return true;
    const Bf16Plan pl = plan_bf16(ci, co, ks, g);
    if (!pl.ok) return false;
    Bf16Args a{};
    a.in = in.p; a.isn = in.sn; a.isc = in.sc;
    a.scale_shift = scale_shift;
    a.w = w;
    a.wq = wq; a.CIP = (ci + 7) / 8 * 8;
    a.r = r ? r->p : nullptr; a.rsn = r ? r->sn : 0; a.rsc = r ? r->sc : 0;
    a.out = out.p; a.osn = out.sn; a.osc = out.sc;
    a.N = g.n; a.H = g.h; a.W = g.w; a.CI = ci; a.CO = co;
    a.ep = (int)ep; a.transposed = transposed ? 1 : 0;
    a.TR = pl.TR; a.IMGS = pl.IMGS; a.bands = pl.bands;
    a.pix_per_img = pl.TR * g.w; a.n_pix = pl.IMGS * pl.TR * g.w;
    a.lrows = pl.lrows; a.lcols = pl.lcols; a.Wq = pl.Wq; a.in_items = pl.in_items;
    const dim3 grid((unsigned)(pl.bands * ((g.n + pl.IMGS - 1) / pl.IMGS)), (unsigned)((co + pl.MT * 32 - 1) / (pl.MT * 32)));
#define RVN_CASE(KS_, MT_, NT_, KC_)                                                                     \
    if (ks == KS_ && pl.MT == MT_ && pl.NT == NT_ && pl.KC == KC_) {                                     \
        cx.run(conv_bf16_k<KS_, MT_, NT_, KC_>, grid, dim3(kThreads), pl.lds_bytes, a);                  \
        return true;                                                                                     \
    }
#define RVN_CASES(KS_, KC_)                                                                              \
    RVN_CASE(KS_, 1, 1, KC_) RVN_CASE(KS_, 1, 2, KC_) RVN_CASE(KS_, 1, 4, KC_)                           \
    RVN_CASE(KS_, 2, 1, KC_) RVN_CASE(KS_, 2, 2, KC_) RVN_CASE(KS_, 4, 1, KC_)
    RVN_CASES(3, 16) RVN_CASES(3, 32) RVN_CASES(3, 64) RVN_CASES(1, 16) RVN_CASES(1, 32) RVN_CASES(1, 64) RVN_CASES(1, 128)
#undef RVN_CASES
#undef RVN_CASE
    return false;
}

}  // namespace rvn
