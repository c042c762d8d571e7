// Fixed-point residual stream (Section 3.2, "Numerical error": with the x's
// and y's in fixed point and F, G in ordinary floating point, the additive
// coupling is undone exactly).  A stream element is an int32 code q standing
// for q * 2^-frac_bits.  Two streaming kernels connect it to the floating-point
// residual functions:
//   fix_to_float:  xf = float(q) * 2^-frac_bits           (the function's input)
//   fix_axpy:      out = r + sign * rint(f * 2^frac_bits)  (y = x + F, x = y - F)
// The sum is an integer sum, so subtracting the same rint(f * 2^frac_bits)
// returns r bit for bit; f is the same when the function is evaluated again on
// the same input, because the kernels are deterministic.
#include "kernels.h"

namespace rvn {

namespace {

constexpr int kThreads = 256;

// One thread per element (quads if VEC); planes of HW elements, strided source / destination.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void fix_to_float_k(const int *__restrict__ x, int64_t sn, int64_t sc,
                                                           float *__restrict__ out, int C, int per, float unit,
                                                           int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int e = (int)(i % per);
    const int64_t plane = i / per;
    const int c = (int)(plane % C);
    const int64_t n = plane / C;
    const int *src = x + n * sn + (int64_t)c * sc;
    if (VEC) {
        const int4 q = reinterpret_cast<const int4 *>(src)[e];
        reinterpret_cast<float4 *>(out)[i] = make_float4((float)q.x * unit, (float)q.y * unit, (float)q.z * unit, (float)q.w * unit);
    } else {
        out[i] = (float)src[e] * unit;
    }
}

// q + sign * rint(v) on codes.  The documented behaviour on overflow is wrap-around, so the sum is
// formed in unsigned arithmetic (signed overflow would be undefined); the conversion of v saturates.
__device__ __forceinline__ int code_axpy(int q, int sign, float v) {
    const uint32_t t = (uint32_t)__float2int_rn(v);
    return (int)(sign > 0 ? (uint32_t)q + t : (uint32_t)q - t);
}

// out = r + sign * rint(f * scale); f dense, r and out strided; out may be r.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void fix_axpy_k(const int *r, int64_t rsn, int64_t rsc, const float *__restrict__ f,
                                                       int *out, int64_t osn, int64_t osc, int C, int per, float scale,
                                                       int sign, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int e = (int)(i % per);
    const int64_t plane = i / per;
    const int c = (int)(plane % C);
    const int64_t n = plane / C;
    const int *rp = r + n * rsn + (int64_t)c * rsc;
    int *op = out + n * osn + (int64_t)c * osc;
    if (VEC) {
        const int4 q = reinterpret_cast<const int4 *>(rp)[e];
        const float4 v = reinterpret_cast<const float4 *>(f)[i];
        int4 o;
        o.x = code_axpy(q.x, sign, v.x * scale);
        o.y = code_axpy(q.y, sign, v.y * scale);
        o.z = code_axpy(q.z, sign, v.z * scale);
        o.w = code_axpy(q.w, sign, v.w * scale);
        reinterpret_cast<int4 *>(op)[e] = o;
    } else {
        op[e] = code_axpy(rp[e], sign, f[i] * scale);
    }
}

// q = rint(x * scale), both strided (entry into the fixed-point stream).
__global__ __launch_bounds__(kThreads) void fix_from_float_k(const float *__restrict__ x, int64_t sn, int64_t sc,
                                                             int *__restrict__ out, int64_t osn, int64_t osc, int C, int HW,
                                                             float scale, int64_t total) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= total) return;
    const int e = (int)(i % HW);
    const int64_t plane = i / HW;
    const int c = (int)(plane % C);
    const int64_t n = plane / C;
    out[n * osn + (int64_t)c * osc + e] = __float2int_rn(x[n * sn + (int64_t)c * sc + e] * scale);
}

bool aligned16(const View &v, int hw) {
    return hw % 4 == 0 && v.sn % 4 == 0 && v.sc % 4 == 0 && (reinterpret_cast<uintptr_t>(v.p) & 15) == 0;
}

unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }

}  // namespace

void fix_to_float(Ctx &cx, View x, int c, Geo g, int frac_bits, float *out) {
    const int64_t elems = g.pixels() * c;
    if (!cx.launch(K_FIXED_POINT, 8.0 * (double)elems)) return;
    const float unit = ldexpf(1.0f, -frac_bits);
    const int *xp = reinterpret_cast<const int *>(x.p);
    if (aligned16(x, g.hw()) && (reinterpret_cast<uintptr_t>(out) & 15) == 0)
        cx.run(fix_to_float_k<true>, dim3(blocks_for(elems / 4)), dim3(kThreads), 0, xp, x.sn, x.sc, out, c, g.hw() / 4, unit, elems / 4);
    else
        cx.run(fix_to_float_k<false>, dim3(blocks_for(elems)), dim3(kThreads), 0, xp, x.sn, x.sc, out, c, g.hw(), unit, elems);
}

void fix_axpy(Ctx &cx, View r, const float *f, int c, Geo g, int frac_bits, int sign, View out) {
    const int64_t elems = g.pixels() * c;
    if (!cx.launch(K_FIXED_POINT, 12.0 * (double)elems)) return;
    const float scale = ldexpf(1.0f, frac_bits);
    const int *rp = reinterpret_cast<const int *>(r.p);
    int *op = reinterpret_cast<int *>(out.p);
    if (aligned16(r, g.hw()) && aligned16(out, g.hw()) && (reinterpret_cast<uintptr_t>(f) & 15) == 0)
        cx.run(fix_axpy_k<true>, dim3(blocks_for(elems / 4)), dim3(kThreads), 0, rp, r.sn, r.sc, f, op, out.sn, out.sc, c,
               g.hw() / 4, scale, sign, elems / 4);
    else
        cx.run(fix_axpy_k<false>, dim3(blocks_for(elems)), dim3(kThreads), 0, rp, r.sn, r.sc, f, op, out.sn, out.sc, c, g.hw(),
               scale, sign, elems);
}

void fix_from_float(Ctx &cx, View x, int c, Geo g, int frac_bits, View out) {
    const int64_t elems = g.pixels() * c;
    if (!cx.launch(K_FIXED_POINT, 8.0 * (double)elems)) return;
    cx.run(fix_from_float_k, dim3(blocks_for(elems)), dim3(kThreads), 0, (const float *)x.p, x.sn, x.sc,
           reinterpret_cast<int *>(out.p), out.sn, out.sc, c, g.hw(), ldexpf(1.0f, frac_bits), elems);
}

}  // namespace rvn
