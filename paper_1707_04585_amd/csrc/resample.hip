// Elementwise helpers of the non-reversible subsampling block (Section 3.1:
// reversible blocks have stride 1, so ordinary stride-2 layers sit between the
// stages).  A stride-2 convolution with padding (k-1)/2 on an even-sized image
// is every second row and column of the stride-1 convolution, and its two
// adjoints are the stride-1 adjoints of the output gradient spread out with
// zeros in between; these kernels do the taking and the spreading, the
// convolutions themselves run on the stride-1 matrix-core kernels.
//
// All three are pure HBM streaming: one thread per low-resolution quad
// (subsample) or per full-resolution quad of one row (the two upsamplers),
// 16-byte accesses on the dense side.
#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;

// out[n][c][p][q] = in[n][c][2p][2q]; out dense [n][c][h/2][w/2].
__global__ __launch_bounds__(kThreads) void subsample2_k(const float *__restrict__ in, int64_t isn, int64_t isc,
                                                         float *__restrict__ out, int C, int H2, int W2,
                                                         int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int q = (int)(i % W2);
    int64_t t = i / W2;
    const int p = (int)(t % H2);
    t /= H2;
    const int c = (int)(t % C);
    const int64_t n = t / C;
    out[i] = in[n * isn + (int64_t)c * isc + (int64_t)(2 * p) * (2 * W2) + 2 * q];
}

// out[n][c][i][j] = (i, j both even) ? in[n][c][i/2][j/2] : 0, both dense; one
// thread per output pair (j, j+1), j even.
__global__ __launch_bounds__(kThreads) void upsample2_zero_k(const float *__restrict__ in, float *__restrict__ out,
                                                             int H2, int W2, int64_t pairs) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= pairs) return;
    const int q = (int)(i % W2);
    int64_t t = i / W2;
    const int row = (int)(t % (2 * H2));
    const int64_t plane = t / (2 * H2);
    float2 v = {0.f, 0.f};
    if ((row & 1) == 0) v.x = in[(plane * H2 + (row >> 1)) * W2 + q];
    reinterpret_cast<float2 *>(out)[i] = v;
}

// acc[n][c][2p][2q] += t[n][c][p][q], both dense.
__global__ __launch_bounds__(kThreads) void upsample2_add_k(const float *__restrict__ t, float *__restrict__ acc,
                                                            int H2, int W2, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int q = (int)(i % W2);
    int64_t r = i / W2;
    const int p = (int)(r % H2);
    const int64_t plane = r / H2;
    float *d = acc + ((plane * (2 * H2) + 2 * p) * (int64_t)(2 * W2)) + 2 * q;
    *d += t[i];
}

unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

}  // namespace

void subsample2(Ctx &cx, View in, int c, Geo full, float *out) {
    const int h2 = full.h / 2, w2 = full.w / 2;
    const int64_t total = (int64_t)full.n * c * h2 * w2;
    if (!cx.launch(K_RESAMPLE, 8.0 * (double)total)) return;
    cx.run(subsample2_k, dim3(blocks_for(total)), dim3(kThreads), 0, (const float *)in.p, in.sn, in.sc, out, c, h2, w2, total);
}

void upsample2_zero(Ctx &cx, const float *in, int c, Geo full, float *out) {
    const int h2 = full.h / 2, w2 = full.w / 2;
    const int64_t pairs = (int64_t)full.n * c * full.h * w2;
    if (!cx.launch(K_RESAMPLE, 4.0 * (double)full.n * c * h2 * w2 + 8.0 * (double)pairs)) return;
    cx.run(upsample2_zero_k, dim3(blocks_for(pairs)), dim3(kThreads), 0, in, out, h2, w2, pairs);
}

void upsample2_add(Ctx &cx, const float *t, int c, Geo full, float *acc) {
    const int h2 = full.h / 2, w2 = full.w / 2;
    const int64_t total = (int64_t)full.n * c * h2 * w2;
    if (!cx.launch(K_RESAMPLE, 12.0 * (double)total)) return;
    cx.run(upsample2_add_k, dim3(blocks_for(total)), dim3(kThreads), 0, t, acc, h2, w2, total);
}

}  // namespace rvn
