// Train-mode batch normalisation + ReLU, forward and backward, for gfx950.
//
// a(x) = ReLU(BN(x)) is the first half of every unit c_k(x) = Conv(a(x)) of
// the residual functions (Section 2.2).  All kernels here are bound by HBM
// bandwidth: each streams whole [n][c][h*w] tensors once with 16-byte
// accesses and reduces per channel with wavefront shuffles and LDS.  The
// cross-workgroup part of a reduction is finished by the workgroup that
// arrives last at a per-channel ticket counter; the merge itself runs in a
// fixed order (no floating-point atomics), so results are bitwise
// reproducible -- the reconstruction of Section 3.2 relies on recomputing
// exactly what the forward pass computed.
#include "kernels.h"
#include "prep_filter.h"
#include "wgrad_reduce.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
    return v;
}

// Sum NV values over the 256 threads of a workgroup; result in thread 0.
template <int NV>
__device__ __forceinline__ void block_sum(float (&v)[NV], float *lds) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < NV; ++i) v[i] = wave_sum(v[i]);
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i) lds[wave * NV + i] = v[i];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
            v[i] = (lds[i] + lds[NV + i]) + (lds[2 * NV + i] + lds[3 * NV + i]);
    }
}

// Partial results cross workgroups (and XCDs, whose L2s are not coherent with
// each other inside a kernel) through device-scope accesses: a device-scope
// store is written through to the memory side, a device-scope load is served
// from there.  That avoids device-scope fences, which write back and
// invalidate a whole L2 each time.
__device__ __forceinline__ void publish(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float fetch(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Ticket: thread 0 (which has publish()ed this workgroup's partial result)
// waits until those stores have completed and takes a ticket; the workgroup
// holding the last of `expected` tickets returns true for all its threads and
// has put the counter back to zero for the next use.  It must read the other
// workgroups' results with fetch().
//
// The wait is explicit.  A workgroup-scope release fence only keeps the
// compiler from moving the stores; it emits no s_waitcnt, and a store and an
// atomic to different addresses travel to different L2 channels, so without
// the wait the ticket can overtake the partial result and the last workgroup
// can fetch what an earlier launch left there.  (An agent-scope fence would
// wait as well, but it also writes back the whole L2.)
__device__ __forceinline__ void wait_for_own_stores() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): every vector memory operation of this thread has completed
}

__device__ __forceinline__ bool arrive_last(int *counter, int expected, int *flag_lds) {
    if (threadIdx.x == 0) {
        wait_for_own_stores();
        const int prev = atomicAdd(counter, 1);
        const int last = prev == expected - 1;
        if (last) atomicExch(counter, 0);
        *flag_lds = last;
    }
    __syncthreads();
    return *flag_lds != 0;
}

// e / d with a host-made multiplier m = 2^32 / d + 1 (exact while e * d < 2^32;
// the host passes m = 0 when it cannot promise that, and d is divided by then).
__device__ __forceinline__ int idiv(int e, int d, uint32_t m) { return m ? (int)__umulhi((uint32_t)e, m) : e / d; }

constexpr int kFly = 4;  // items a thread requests before it uses the first

__device__ __forceinline__ double shfl_down_f64(double v, int off) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_down(lo, off, 64);
    hi = __shfl_down(hi, off, 64);
    return __hiloint2double(hi, lo);
}

// ---------------------------------------------------------------------------
// statistics: per (channel, image group) shifted sums -> (count, mean, M2);
// the last workgroup of a channel merges them and writes the four per-channel
// arrays mean, rstd, scale, shift.
// ---------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kThreads) void bn_stats_k(const float *__restrict__ x, int64_t sn,
                                                       int64_t sc, int N, int HW, int ipw, uint32_t m_per,
                                                       float *partial, int *counters, float eps,
                                                       const float *__restrict__ gamma,
                                                       const float *__restrict__ beta,
                                                       float *__restrict__ stats, int S, int C,
                                                       const PrepArgs carry) {
    // The first carry.blocks workgroups convert the residual function's filters
    // (independent work that would otherwise be a launch of its own).
    if ((int)blockIdx.x < carry.blocks) {
        prep_filter_body(carry, blockIdx.x);
        return;
    }
    __shared__ float lds[8];
    __shared__ int flag;
    const int lin = blockIdx.x - carry.blocks;
    const int ch = lin / S, s = lin - ch * S;
    const int n0 = s * ipw, n1 = min(N, n0 + ipw);
    const float *base = x + (int64_t)ch * sc;
    // Shift by a value from the data so that the sum of squares does not
    // cancel when |mean| >> std (the residual stream grows with depth).
    const float pivot = base[(int64_t)n0 * sn];
    float acc[2] = {0.f, 0.f};
    // The workgroup's images as one index space (quads if VEC), kFly loads in
    // flight per thread; indices past the end re-read a valid item and add 0.
    const int per = VEC ? HW / 4 : HW, total = (n1 - n0) * per;
    for (int q0 = threadIdx.x; q0 < total; q0 += kFly * kThreads) {
        float4 v[kFly];
        bool ok[kFly];
#pragma unroll
        for (int k = 0; k < kFly; ++k) {
            const int q = q0 + k * kThreads;
            ok[k] = q < total;
            const int qc = ok[k] ? q : q0;
            const int n = idiv(qc, per, m_per), i = qc - n * per;
            const float *pl = base + (int64_t)(n0 + n) * sn;
            if (VEC) {
                v[k] = reinterpret_cast<const float4 *>(pl)[i];
            } else {
                v[k].x = pl[i];
            }
        }
#pragma unroll
        for (int k = 0; k < kFly; ++k) {
            if (VEC) {
                const float a = ok[k] ? v[k].x - pivot : 0.f, b = ok[k] ? v[k].y - pivot : 0.f;
                const float c = ok[k] ? v[k].z - pivot : 0.f, d = ok[k] ? v[k].w - pivot : 0.f;
                acc[0] += (a + b) + (c + d);
                acc[1] += (a * a + b * b) + (c * c + d * d);
            } else {
                const float d = ok[k] ? v[k].x - pivot : 0.f;
                acc[0] += d;
                acc[1] += d * d;
            }
        }
    }
    block_sum<2>(acc, lds);
    if (threadIdx.x == 0) {
        const float cnt = (float)((n1 - n0) * HW);
        float *o = partial + ((int64_t)ch * S + s) * 3;
        publish(o, cnt);
        publish(o + 1, pivot + acc[0] / cnt);
        publish(o + 2, fmaxf(acc[1] - acc[0] * acc[0] / cnt, 0.f));
    }
    if (!arrive_last(counters + ch * kCounterStride, S, &flag)) return;
    // Merge the S <= 64 partials (Chan et al.) in a fixed shuffle tree, in
    // double precision; lane s holds partial s.
    if (threadIdx.x >= 64) return;
    const int lane = threadIdx.x;
    double n = 0.0, mean = 0.0, m2 = 0.0;
    if (lane < S) {
        const float *q = partial + ((int64_t)ch * S + lane) * 3;
        n = fetch(q);
        mean = fetch(q + 1);
        m2 = fetch(q + 2);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const double nb = shfl_down_f64(n, off), mb = shfl_down_f64(mean, off), m2b = shfl_down_f64(m2, off);
        const double tot = n + nb;
        if (tot > 0.0) {
            const double delta = mb - mean, fb = nb / tot;
            mean += delta * fb;
            m2 += m2b + delta * delta * n * fb;
        }
        n = tot;
    }
    if (lane == 0) {
        const float mean_f = (float)mean;
        const float rstd_f = (float)(1.0 / sqrt(m2 / n + (double)eps));
        const float scale = gamma[ch] * rstd_f;
        stats[ch] = mean_f;
        stats[C + ch] = rstd_f;
        stats[2 * C + ch] = scale;
        stats[3 * C + ch] = fmaf(-mean_f, scale, beta[ch]);
    }
}

// ---------------------------------------------------------------------------
// statistics from partial results: (mean, M2) of every pixel tile of a
// channel, written by the convolution that produced the tensor, merged (Chan
// et al., double precision, fixed order) into the same four per-channel arrays.
// One workgroup per channel: thread t takes tiles t, t + 256, ..., then a
// shuffle tree per wavefront and the four wavefronts in order.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void chan_merge(double &n, double &mean, double &m2, double nb, double mb, double m2b) {
    const double tot = n + nb;
    if (tot > 0.0) {
        const double delta = mb - mean, fb = nb / tot;
        mean += delta * fb;
        m2 += m2b + delta * delta * n * fb;
    }
    n = tot;
}

// Channel `ch` of the merge, by one workgroup of kThreads threads.
__device__ __forceinline__ void bn_stats_merge_body(const float *__restrict__ partials, int tiles, float count, float eps,
                                                    const float *__restrict__ gamma, const float *__restrict__ beta,
                                                    float *__restrict__ stats, int C, int ch) {
    __shared__ double red[kThreads / 64][3];
    const float2 *q = reinterpret_cast<const float2 *>(partials) + (int64_t)ch * tiles;
    double n = 0.0, mean = 0.0, m2 = 0.0;
    for (int t0 = threadIdx.x; t0 < tiles; t0 += 8 * kThreads) {
        float2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = q[min(t0 + u * kThreads, tiles - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (t0 + u * kThreads < tiles) chan_merge(n, mean, m2, (double)count, (double)v[u].x, (double)v[u].y);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        chan_merge(n, mean, m2, shfl_down_f64(n, off), shfl_down_f64(mean, off), shfl_down_f64(m2, off));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) red[wave][0] = n, red[wave][1] = mean, red[wave][2] = m2;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int wv = 1; wv < kThreads / 64; ++wv) chan_merge(n, mean, m2, red[wv][0], red[wv][1], red[wv][2]);
        const float mean_f = (float)mean;
        const float rstd_f = (float)(1.0 / sqrt(m2 / n + (double)eps));
        const float scale = gamma[ch] * rstd_f;
        stats[ch] = mean_f;
        stats[C + ch] = rstd_f;
        stats[2 * C + ch] = scale;
        stats[3 * C + ch] = fmaf(-mean_f, scale, beta[ch]);
    }
}

__global__ __launch_bounds__(kThreads) void bn_stats_merge_k(const float *__restrict__ partials, int tiles, float count,
                                                             float eps, const float *__restrict__ gamma,
                                                             const float *__restrict__ beta, float *__restrict__ stats,
                                                             int C, const PrepArgs carry) {
    if ((int)blockIdx.x < carry.blocks) {
        prep_filter_body(carry, blockIdx.x);
        return;
    }
    bn_stats_merge_body(partials, tiles, count, eps, gamma, beta, stats, C, (int)blockIdx.x - carry.blocks);
}

// ---------------------------------------------------------------------------
// backward, reduce pass: per-channel sums of dy and dy*xhat, dy = da * [u > 0];
// the last workgroup of a channel writes dbeta = sum dy, dgamma = sum dy*xhat
// and the two per-channel means the apply pass needs (kept apart from
// dgamma/dbeta, which may be accumulated into).
// ---------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kThreads) void bn_bwd_reduce_k(
    const float *__restrict__ x, int64_t sn, int64_t sc, const float *__restrict__ da, int N, int C,
    int HW, int ipw, uint32_t m_per, const float *__restrict__ stats, float *partial, int *counters, double inv_m,
    float *__restrict__ dgamma, float *__restrict__ dbeta, int accumulate, float *__restrict__ coef) {
    __shared__ float lds[8];
    __shared__ int flag;
    const int ch = blockIdx.y, s = blockIdx.x, S = gridDim.x;
    const int n0 = s * ipw, n1 = min(N, n0 + ipw);
    const float mean = stats[ch], rstd = stats[C + ch];
    const float scale = stats[2 * C + ch], shift = stats[3 * C + ch];
    float acc[2] = {0.f, 0.f};
    const int per = VEC ? HW / 4 : HW, total = (n1 - n0) * per;
    for (int q0 = threadIdx.x; q0 < total; q0 += kFly * kThreads) {
        float4 xv[kFly], dv[kFly];
        bool ok[kFly];
#pragma unroll
        for (int k = 0; k < kFly; ++k) {
            const int q = q0 + k * kThreads;
            ok[k] = q < total;
            const int qc = ok[k] ? q : q0;
            const int n = idiv(qc, per, m_per), i = qc - n * per;
            const float *px = x + (int64_t)(n0 + n) * sn + (int64_t)ch * sc;
            const float *pd = da + ((int64_t)(n0 + n) * C + ch) * HW;
            if (VEC) {
                xv[k] = reinterpret_cast<const float4 *>(px)[i];
                dv[k] = reinterpret_cast<const float4 *>(pd)[i];
            } else {
                xv[k].x = px[i];
                dv[k].x = pd[i];
            }
        }
#pragma unroll
        for (int k = 0; k < kFly; ++k) {
            const float xs[4] = {xv[k].x, xv[k].y, xv[k].z, xv[k].w};
            const float ds[4] = {dv[k].x, dv[k].y, dv[k].z, dv[k].w};
#pragma unroll
            for (int j = 0; j < (VEC ? 4 : 1); ++j) {
                const float dy = ok[k] && fmaf(xs[j], scale, shift) > 0.f ? ds[j] : 0.f;
                acc[0] += dy;
                acc[1] += dy * ((xs[j] - mean) * rstd);
            }
        }
    }
    block_sum<2>(acc, lds);
    if (threadIdx.x == 0) {
        float *o = partial + ((int64_t)ch * S + s) * 2;
        publish(o, acc[0]);
        publish(o + 1, acc[1]);
    }
    if (!arrive_last(counters + ch * kCounterStride, S, &flag)) return;
    if (threadIdx.x >= 64) return;
    const int lane = threadIdx.x;
    double sb = 0.0, sg = 0.0;
    if (lane < S) {
        const float *q = partial + ((int64_t)ch * S + lane) * 2;
        sb = fetch(q);
        sg = fetch(q + 1);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        sb += shfl_down_f64(sb, off);
        sg += shfl_down_f64(sg, off);
    }
    if (lane == 0) {
        if (accumulate) {
            dbeta[ch] += (float)sb;
            dgamma[ch] += (float)sg;
        } else {
            dbeta[ch] = (float)sb;
            dgamma[ch] = (float)sg;
        }
        coef[ch] = (float)(sb * inv_m);
        coef[C + ch] = (float)(sg * inv_m);
    }
}

// dx = gamma*rstd*(dy - mean(dy) - xhat*mean(dy*xhat)); out = [skip +] dx
template <bool VEC, bool SKIP, bool PREP>
__device__ __forceinline__ void bn_bwd_apply_body(
    const float *__restrict__ x, int64_t sn, int64_t sc, const float *da, int C, int HW,
    int64_t total, const float *__restrict__ stats, const float *__restrict__ coef, const float *skip,
    int64_t ksn, int64_t ksc, float *out, int64_t osn, int64_t osc, const WgradReduce &carry, const StatsMerge &merge,
    const PrepArgs &prep, uint16_t *out16) {
    // The first workgroups do independent work that would otherwise be launches of their own (first,
    // so that their dependent loads run under the streaming of the others): merge.blocks of them merge
    // the partial statistics of a tensor that a later BN layer reads, carry.blocks sum a filter
    // gradient's partial results.
    if ((int)blockIdx.x < merge.blocks) {
        bn_stats_merge_body(merge.partials, merge.tiles, merge.count, merge.eps, merge.gamma, merge.beta, merge.stats,
                            merge.C, (int)blockIdx.x);
        return;
    }
    // (and, in the PREP variant, prep.blocks convert the filters of the function that will read those statistics)
    const int prep_blocks = PREP ? prep.blocks : 0;
    if (PREP && (int)blockIdx.x < merge.blocks + prep_blocks) {
        prep_filter_body(prep, (int)blockIdx.x - merge.blocks);
        return;
    }
    const int bx = (int)blockIdx.x - merge.blocks - prep_blocks;
    if (bx < carry.blocks) {
        __shared__ float lds[kThreads];
        wgrad_reduce_body(carry, bx, lds);
        return;
    }
    constexpr int E = VEC ? 4 : 1;
    const int64_t v = (int64_t)(bx - carry.blocks) * kThreads + threadIdx.x;
    if (v >= total) return;
    const int per_plane = HW / E;
    const int64_t plane = v / per_plane;
    const int i = (int)(v - plane * per_plane) * E;
    const int n = (int)(plane / C), ch = (int)(plane - (int64_t)n * C);
    const float mean = stats[ch], rstd = stats[C + ch];
    const float scale = stats[2 * C + ch], shift = stats[3 * C + ch];
    const float c1 = coef[ch], c2 = coef[C + ch];
    const float *px = x + (int64_t)n * sn + (int64_t)ch * sc + i;
    const float *pd = da + plane * HW + i;
    float *po = out + (int64_t)n * osn + (int64_t)ch * osc + i;
    const float *pk = SKIP ? skip + (int64_t)n * ksn + (int64_t)ch * ksc + i : nullptr;
    if (VEC) {
        const float4 xv = *reinterpret_cast<const float4 *>(px);
        const float4 dv = *reinterpret_cast<const float4 *>(pd);
        float4 kv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (SKIP) kv = *reinterpret_cast<const float4 *>(pk);
        const float xs[4] = {xv.x, xv.y, xv.z, xv.w};
        const float ds[4] = {dv.x, dv.y, dv.z, dv.w};
        const float ks[4] = {kv.x, kv.y, kv.z, kv.w};
        float r[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float dy = fmaf(xs[j], scale, shift) > 0.f ? ds[j] : 0.f;
            const float xh = (xs[j] - mean) * rstd;
            const float dx = scale * ((dy - c1) - xh * c2);
            r[j] = SKIP ? ks[j] + dx : dx;
        }
        if (out16) {  // (uniform) dense bf16, nearest even: what the convolutions that read it would round it to
            typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
            typedef float float2_t __attribute__((ext_vector_type(2)));
            const float2_t lo = {r[0], r[1]}, hi = {r[2], r[3]};
            const bf16x2_t blo = __builtin_convertvector(lo, bf16x2_t), bhi = __builtin_convertvector(hi, bf16x2_t);
            *reinterpret_cast<uint2 *>(out16 + plane * HW + i) =
                make_uint2(*reinterpret_cast<const uint32_t *>(&blo), *reinterpret_cast<const uint32_t *>(&bhi));
        } else {
            *reinterpret_cast<float4 *>(po) = make_float4(r[0], r[1], r[2], r[3]);
        }
    } else {
        const float xv = *px;
        const float dy = fmaf(xv, scale, shift) > 0.f ? *pd : 0.f;
        const float xh = (xv - mean) * rstd;
        const float dx = scale * ((dy - c1) - xh * c2);
        *po = SKIP ? *pk + dx : dx;
    }
}

template <bool VEC, bool SKIP>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_k(
    const float *__restrict__ x, int64_t sn, int64_t sc, const float *da, int C, int HW,
    int64_t total, const float *__restrict__ stats, const float *__restrict__ coef, const float *skip,
    int64_t ksn, int64_t ksc, float *out, int64_t osn, int64_t osc, const WgradReduce carry, const StatsMerge merge,
    uint16_t *out16) {
    bn_bwd_apply_body<VEC, SKIP, false>(x, sn, sc, da, C, HW, total, stats, coef, skip, ksn, ksc, out, osn, osc, carry,
                                        merge, PrepArgs{}, out16);
}

// The same with a filter conversion among the carried work (a large argument block: kept out of the
// ordinary launches).
template <bool VEC, bool SKIP>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply_prep_k(
    const float *__restrict__ x, int64_t sn, int64_t sc, const float *da, int C, int HW,
    int64_t total, const float *__restrict__ stats, const float *__restrict__ coef, const float *skip,
    int64_t ksn, int64_t ksc, float *out, int64_t osn, int64_t osc, const WgradReduce carry, const StatsMerge merge,
    const PrepArgs prep) {
    bn_bwd_apply_body<VEC, SKIP, true>(x, sn, sc, da, C, HW, total, stats, coef, skip, ksn, ksc, out, osn, osc, carry,
                                       merge, prep, nullptr);
}

// Both passes in one launch, for layers whose channels are small: one workgroup per channel keeps the
// channel's x and da in registers (at most kFusedQuads 16-byte quads per thread), sums, and applies --
// x and da are read once, and there is no ticket and no second launch.  (Aligned planes of whole quads
// only; the sums are formed per thread, then per wavefront, then over the four wavefronts, in double
// from the wavefront sums on: a fixed order.)
// (For larger channels a two-loop form of the same -- second loop from L2 -- measured slower than the two
// launches: 21.8 against 8.0 + 12.0 us at 128 channels of 28x28 x 32 images, 15.3 against 5.5 + 5.7 us at
// 32 channels of 16x16 x 128: one workgroup per channel is then too little parallelism.)
constexpr int kFusedQuads = 8;

// VEC: aligned planes of whole 4-pixel quads (16-byte accesses); otherwise element by element (7x7 planes;
// channels of at most 2048 elements then: with 32 items per thread the launch was slower than two).
template <bool SKIP, bool PREP, bool VEC>
__device__ __forceinline__ void bn_bwd_fused_body(
    const float *__restrict__ x, int64_t sn, int64_t sc, const float *da, int N, int C, int HW, uint32_t m_per,
    const float *__restrict__ stats, double inv_m, float *__restrict__ dgamma, float *__restrict__ dbeta,
    int accumulate, const float *skip, int64_t ksn, int64_t ksc, float *out, int64_t osn, int64_t osc, uint16_t *out16,
    const WgradReduce &carry, const StatsMerge &merge, const PrepArgs &prep) {
    // carried work first, as in bn_bwd_apply_body
    if ((int)blockIdx.x < merge.blocks) {
        bn_stats_merge_body(merge.partials, merge.tiles, merge.count, merge.eps, merge.gamma, merge.beta, merge.stats,
                            merge.C, (int)blockIdx.x);
        return;
    }
    const int prep_blocks = PREP ? prep.blocks : 0;
    if (PREP && (int)blockIdx.x < merge.blocks + prep_blocks) {
        prep_filter_body(prep, (int)blockIdx.x - merge.blocks);
        return;
    }
    const int bx = (int)blockIdx.x - merge.blocks - prep_blocks;
    if (bx < carry.blocks) {
        __shared__ float lds[kThreads];
        wgrad_reduce_body(carry, bx, lds);
        return;
    }
    __shared__ double sums[8];
    constexpr int E = VEC ? 4 : 1, K = kFusedQuads;  // elements per item, items per thread
    const int ch = bx - carry.blocks;
    const int per = HW / E, total = N * per;
    const float mean = stats[ch], rstd = stats[C + ch];
    const float scale = stats[2 * C + ch], shift = stats[3 * C + ch];
    float xs[K][E], ds[K][E];
    int nn[K], ii[K];  // image and first pixel of the item
    bool ok[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int q = (int)threadIdx.x + k * kThreads;
        ok[k] = q < total;
        const int qc = ok[k] ? q : 0;
        nn[k] = idiv(qc, per, m_per);
        ii[k] = (qc - nn[k] * per) * E;
        const float *px = x + (int64_t)nn[k] * sn + (int64_t)ch * sc + ii[k];
        const float *pd = da + ((int64_t)nn[k] * C + ch) * HW + ii[k];
        if constexpr (VEC) {
            const float4 xv = *reinterpret_cast<const float4 *>(px), dv = *reinterpret_cast<const float4 *>(pd);
            xs[k][0] = xv.x; xs[k][1] = xv.y; xs[k][2] = xv.z; xs[k][3] = xv.w;
            ds[k][0] = dv.x; ds[k][1] = dv.y; ds[k][2] = dv.z; ds[k][3] = dv.w;
        } else {
            xs[k][0] = *px;
            ds[k][0] = *pd;
        }
    }
    float a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const float dyv = ok[k] && fmaf(xs[k][j], scale, shift) > 0.f ? ds[k][j] : 0.f;
            const float xhv = (xs[k][j] - mean) * rstd;
            ds[k][j] = dyv;  // from here on: dy and xhat
            xs[k][j] = xhv;
            a0 += dyv;
            a1 += dyv * xhv;
        }
    }
    a0 = wave_sum(a0);
    a1 = wave_sum(a1);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        sums[wave * 2] = (double)a0;
        sums[wave * 2 + 1] = (double)a1;
    }
    __syncthreads();
    const double sb = (sums[0] + sums[2]) + (sums[4] + sums[6]), sg = (sums[1] + sums[3]) + (sums[5] + sums[7]);
    if (threadIdx.x == 0) {
        if (accumulate) {
            dbeta[ch] += (float)sb;
            dgamma[ch] += (float)sg;
        } else {
            dbeta[ch] = (float)sb;
            dgamma[ch] = (float)sg;
        }
    }
    const float c1 = (float)(sb * inv_m), c2 = (float)(sg * inv_m);
#pragma unroll
    for (int k = 0; k < K; ++k) {
        if (!ok[k]) continue;
        float r[E];
#pragma unroll
        for (int j = 0; j < E; ++j) r[j] = scale * ((ds[k][j] - c1) - xs[k][j] * c2);
        const int n = nn[k], i = ii[k];
        float *po = out + (int64_t)n * osn + (int64_t)ch * osc + i;
        if constexpr (VEC) {
            if (SKIP) {
                const float4 kv = *reinterpret_cast<const float4 *>(skip + (int64_t)n * ksn + (int64_t)ch * ksc + i);
                r[0] += kv.x; r[1] += kv.y; r[2] += kv.z; r[3] += kv.w;
                *reinterpret_cast<float4 *>(po) = make_float4(r[0], r[1], r[2], r[3]);
            } else if (out16) {  // (uniform) dense bf16, nearest even
                typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
                typedef float float2_t __attribute__((ext_vector_type(2)));
                const float2_t lo = {r[0], r[1]}, hi = {r[2], r[3]};
                const bf16x2_t blo = __builtin_convertvector(lo, bf16x2_t), bhi = __builtin_convertvector(hi, bf16x2_t);
                *reinterpret_cast<uint2 *>(out16 + ((int64_t)n * C + ch) * HW + i) =
                    make_uint2(*reinterpret_cast<const uint32_t *>(&blo), *reinterpret_cast<const uint32_t *>(&bhi));
            } else {
                *reinterpret_cast<float4 *>(po) = make_float4(r[0], r[1], r[2], r[3]);
            }
        } else {
            *po = SKIP ? skip[(int64_t)n * ksn + (int64_t)ch * ksc + i] + r[0] : r[0];
        }
    }
}

template <bool SKIP, bool VEC>
__global__ __launch_bounds__(kThreads) void bn_bwd_fused_k(
    const float *__restrict__ x, int64_t sn, int64_t sc, const float *da, int N, int C, int HW, uint32_t m_per,
    const float *__restrict__ stats, double inv_m, float *__restrict__ dgamma, float *__restrict__ dbeta,
    int accumulate, const float *skip, int64_t ksn, int64_t ksc, float *out, int64_t osn, int64_t osc, uint16_t *out16,
    const WgradReduce carry, const StatsMerge merge) {
    bn_bwd_fused_body<SKIP, false, VEC>(x, sn, sc, da, N, C, HW, m_per, stats, inv_m, dgamma, dbeta, accumulate, skip, ksn,
                                        ksc, out, osn, osc, out16, carry, merge, PrepArgs{});
}

template <bool SKIP, bool VEC>
__global__ __launch_bounds__(kThreads) void bn_bwd_fused_prep_k(
    const float *__restrict__ x, int64_t sn, int64_t sc, const float *da, int N, int C, int HW, uint32_t m_per,
    const float *__restrict__ stats, double inv_m, float *__restrict__ dgamma, float *__restrict__ dbeta,
    int accumulate, const float *skip, int64_t ksn, int64_t ksc, float *out, int64_t osn, int64_t osc,
    const WgradReduce carry, const StatsMerge merge, const PrepArgs prep) {
    bn_bwd_fused_body<SKIP, true, VEC>(x, sn, sc, da, N, C, HW, m_per, stats, inv_m, dgamma, dbeta, accumulate, skip, ksn, ksc,
                                       out, osn, osc, nullptr, carry, merge, prep);
}

__global__ void clear_counters_k(int *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

inline bool vec_ok(const View &v, int hw) {
    return hw % 4 == 0 && v.sn % 4 == 0 && v.sc % 4 == 0 && (reinterpret_cast<uintptr_t>(v.p) & 15) == 0;
}

// Multiplier for idiv: indices run up to images * per, and the shortcut is
// exact while index * per < 2^32.
uint32_t div_magic(int images, int per) {
    if (per <= 1) return 0u;
    if ((uint64_t)images * per * per >= (1ull << 32)) return 0u;
    return (uint32_t)((1ull << 32) / (uint64_t)per + 1ull);
}

}  // namespace

int reduce_splits(int c, const Geo &g) {
    int target = c >= 1024 ? 1 : 1024 / c;
    if (target > 64) target = 64;  // the finishing workgroup merges one partial per lane
    const int s_max = g.n < target ? g.n : target;
    const int ipw = (g.n + s_max - 1) / s_max;
    return (g.n + ipw - 1) / ipw;
}

// Scratch layout (floats): [c*S*3 partials][2c per-channel means for the apply pass].
size_t bn_scratch_floats(int c, const Geo &g) {
    return (size_t)c * reduce_splits(c, g) * 3 + 2 * (size_t)c;
}

void clear_counters(Ctx &cx, int *counters, int n) {
    if (!cx.launch(K_CLEAR_COUNTERS, 0.0)) return;
    cx.run(clear_counters_k, dim3((n + 255) / 256), dim3(256), 0, counters, n);
}

void bn_stats(Ctx &cx, View x, int c, Geo g, float eps, const float *gamma, const float *beta, float *scratch,
              int *counters, float *stats, const PrepArgs *carry, double carry_bytes) {
    // The convolution that wrote x may have left per-tile statistics of exactly this tensor.
    const EmittedStats e = cx.emitted;
    cx.emitted = EmittedStats{};
    if (e.p && cx.emit_buf && e.p == x.p && e.sn == x.sn && e.sc == x.sc && e.c == c && e.n == g.n && e.h == g.h &&
        e.w == g.w) {
        if (!cx.launch(K_BN_STATS, 8.0 * (double)c * e.tiles + carry_bytes)) return;
        PrepArgs pa{};
        if (carry) pa = *carry;
        cx.run(bn_stats_merge_k, dim3((unsigned)(c + pa.blocks)), dim3(kThreads), 0, (const float *)cx.emit_buf, e.tiles,
               (float)e.count, eps, gamma, beta, stats, c, pa);
        return;
    }
    const int S = reduce_splits(c, g);
    const int ipw = (g.n + S - 1) / S;
    if (!cx.launch(K_BN_STATS, 4.0 * (double)g.pixels() * c + carry_bytes)) return;
    PrepArgs pa{};
    if (carry) pa = *carry;
    const dim3 grid((unsigned)(S * c + pa.blocks));
    if (vec_ok(x, g.hw()))
        cx.run(bn_stats_k<true>, grid, dim3(kThreads), 0, x.p, x.sn, x.sc, g.n, g.hw(), ipw, div_magic(ipw, g.hw() / 4), scratch, counters, eps, gamma, beta, stats, S, c, pa);
    else
        cx.run(bn_stats_k<false>, grid, dim3(kThreads), 0, x.p, x.sn, x.sc, g.n, g.hw(), ipw, div_magic(ipw, g.hw()), scratch, counters, eps, gamma, beta, stats, S, c, pa);
}

void bn_relu_bwd(Ctx &cx, View x, const float *da, int c, Geo g, const float *stats, float *scratch,
                 int *counters, float *dgamma, float *dbeta, bool accumulate, const View *skip, View out,
                 const WgradReduce *carry, uint16_t *out16) {
    const int S = reduce_splits(c, g);
    const int ipw = (g.n + S - 1) / S;
    const double t = 4.0 * (double)g.pixels() * c;
    float *coef = scratch + (size_t)c * S * 3;
    const bool vec_in = vec_ok(x, g.hw()) && (reinterpret_cast<uintptr_t>(da) & 15) == 0;
    if (out16 && (skip || !vec_in || cx.carry_now)) {  // a caller's mistake: nothing sensible to launch
        cx.fail(hipErrorInvalidValue);
        return;
    }
    // Small channels: both passes in one launch.
    const bool vec_all = vec_in && (out16 || vec_ok(out, g.hw())) && (!skip || vec_ok(*skip, g.hw()));
    const int64_t items = vec_all ? (int64_t)g.n * (g.hw() / 4) : (int64_t)g.n * g.hw();
    if (items <= (int64_t)kFusedQuads * kThreads) {
        if (cx.launch(K_BN_BWD_APPLY, (skip ? 4.0 : out16 ? 2.5 : 3.0) * t)) {
            WgradReduce red{};
            if (carry) red = *carry;
            if (red.blocks < 0) red.blocks = 0;
            // a waiting merge and filter conversion ride along when the caller says this is the launch
            StatsMerge merge{};
            PrepArgs prep{};
            if (cx.carry_now) {
                merge = cx.merge_carry;
                prep = cx.prep_carry;
                cx.merge_carry = StatsMerge{};
                cx.prep_carry = PrepArgs{};
            }
            const dim3 grid((unsigned)(c + red.blocks + merge.blocks + prep.blocks));
            const double inv_m = 1.0 / (double)g.pixels();
            const uint32_t m_per = div_magic(g.n, vec_all ? g.hw() / 4 : g.hw());
            const float *kp = skip ? skip->p : nullptr;
            const int64_t ksn = skip ? skip->sn : 0, ksc = skip ? skip->sc : 0;
#define RVN_LAUNCH(K, V)                                                                                                 \
    do {                                                                                                                 \
        if (prep.blocks > 0)                                                                                             \
            cx.run(bn_bwd_fused_prep_k<K, V>, grid, dim3(kThreads), 0, x.p, x.sn, x.sc, da, g.n, c, g.hw(), m_per, stats, \
                   inv_m, dgamma, dbeta, accumulate ? 1 : 0, kp, ksn, ksc, out.p, out.sn, out.sc, red, merge, prep);      \
        else                                                                                                             \
            cx.run(bn_bwd_fused_k<K, V>, grid, dim3(kThreads), 0, x.p, x.sn, x.sc, da, g.n, c, g.hw(), m_per, stats,      \
                   inv_m, dgamma, dbeta, accumulate ? 1 : 0, kp, ksn, ksc, out.p, out.sn, out.sc, out16, red, merge);     \
    } while (0)
            if (skip && vec_all) RVN_LAUNCH(true, true);
            else if (skip) RVN_LAUNCH(true, false);
            else if (vec_all) RVN_LAUNCH(false, true);
            else RVN_LAUNCH(false, false);
#undef RVN_LAUNCH
        }
        return;
    }
    if (cx.launch(K_BN_BWD_REDUCE, 2.0 * t)) {
        dim3 grid(S, c);
        const double inv_m = 1.0 / (double)g.pixels();
        if (vec_in)
            cx.run(bn_bwd_reduce_k<true>, grid, dim3(kThreads), 0, x.p, x.sn, x.sc, da, g.n, c, g.hw(), ipw, div_magic(ipw, g.hw() / 4), stats, scratch, counters, inv_m, dgamma, dbeta, accumulate ? 1 : 0, coef);
        else
            cx.run(bn_bwd_reduce_k<false>, grid, dim3(kThreads), 0, x.p, x.sn, x.sc, da, g.n, c, g.hw(), ipw, div_magic(ipw, g.hw()), stats, scratch, counters, inv_m, dgamma, dbeta, accumulate ? 1 : 0, coef);
    }
    if (cx.launch(K_BN_BWD_APPLY, (skip ? 4.0 : out16 ? 2.5 : 3.0) * t)) {
        const bool vec = vec_in && (out16 || vec_ok(out, g.hw())) && (!skip || vec_ok(*skip, g.hw()));
        const int64_t total = (int64_t)g.n * c * (g.hw() / (vec ? 4 : 1));
        const unsigned blocks = (unsigned)((total + kThreads - 1) / kThreads);
        const float *kp = skip ? skip->p : nullptr;
        const int64_t ksn = skip ? skip->sn : 0, ksc = skip ? skip->sc : 0;
        WgradReduce red{};
        if (carry) red = *carry;
        if (red.blocks < 0) red.blocks = 0;
        // a waiting merge and filter conversion ride along when the caller says this is the launch
        StatsMerge merge{};
        PrepArgs prep{};
        if (cx.carry_now) {
            merge = cx.merge_carry;
            prep = cx.prep_carry;
            cx.merge_carry = StatsMerge{};
            cx.prep_carry = PrepArgs{};
        }
        const unsigned extra = (unsigned)red.blocks + (unsigned)merge.blocks + (unsigned)prep.blocks;
#define RVN_LAUNCH(V, K)                                                                                              \
    do {                                                                                                              \
        if (prep.blocks > 0)                                                                                          \
            cx.run(bn_bwd_apply_prep_k<V, K>, dim3(blocks + extra), dim3(kThreads), 0, x.p, x.sn, x.sc, da, c, g.hw(), \
                   total, stats, coef, kp, ksn, ksc, out.p, out.sn, out.sc, red, merge, prep);                         \
        else                                                                                                          \
            cx.run(bn_bwd_apply_k<V, K>, dim3(blocks + extra), dim3(kThreads), 0, x.p, x.sn, x.sc, da, c, g.hw(),      \
                   total, stats, coef, kp, ksn, ksc, out.p, out.sn, out.sc, red, merge, out16);                        \
    } while (0)
        if (vec && skip) RVN_LAUNCH(true, true);
        else if (vec) RVN_LAUNCH(true, false);
        else if (skip) RVN_LAUNCH(false, true);
        else RVN_LAUNCH(false, false);
#undef RVN_LAUNCH
    }
}

}  // namespace rvn
