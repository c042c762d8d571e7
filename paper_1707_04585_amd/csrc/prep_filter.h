// Conversion of a residual function's filters to bf16 in the order the
// convolution kernels consume them, as a body that any launch can carry (a
// launch of its own in conv_bf16.hip, or extra workgroups of the first
// statistics kernel of the function).  Device code only.
#pragma once

#include "kernels.h"

namespace rvn {

// Workgroup `block` (0 .. p.blocks - 1, 256 threads) of the conversion.  A job
// is one destination buffer:
//   kind 0: q[ko][tap][c]  = w[ko][c][tap]           (forward, channel pitch KP)
//   kind 1: q[c][tap][ko]  = w[ko][c][k*k-1-tap]     (data gradient: transposed and flipped, pitch KP)
//   kind 2: q[mt][ks][lane][e] = w[row][col]         (1x1 forward, operand order of conv1x1_bf16:
//   kind 3: q[mt][ks][lane][e] = w[col][row]          row = mt*32 + lane%32, col = ks*16 + (lane/32)*8 + e)
// with zeros outside the filter.
__device__ __forceinline__ void prep_filter_body(const PrepArgs &p, int block) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float float2_t __attribute__((ext_vector_type(2)));
    int j = 0;
#pragma unroll
    for (int i = 1; i < 6; ++i)
        if (i < p.jobs && block >= p.job[i].block0) j = i;
    const PrepJob &jb = p.job[j];
    const int64_t i = (int64_t)(block - jb.block0) * 256 + threadIdx.x;
    if (i >= jb.n) return;
    const int CO = jb.CO, CI = jb.CI, KS2 = jb.KS2;
    auto to_bf16 = [](float v) {  // nearest-even: v_cvt_pk_bf16_f32
        const float2_t f2 = {v, 0.f};
        const bf16x2_t b2 = __builtin_convertvector(f2, bf16x2_t);
        return (uint16_t)(*reinterpret_cast<const uint32_t *>(&b2) & 0xffffu);
    };
    if (jb.kind <= 1) {
        // One thread per (row, padded column) pair and all k*k taps: the taps of a
        // pair are contiguous in w, and neighbouring threads write neighbouring
        // columns of q.
        const int col = (int)(i % jb.KP), row = (int)(i / jb.KP);
        const bool in = jb.kind == 0 ? col < CI : col < CO;
        const float *src = jb.kind == 0 ? jb.w + ((int64_t)row * CI + col) * KS2   // row = ko, col = c
                                        : jb.w + ((int64_t)col * CI + row) * KS2;  // row = c, col = ko
        // All taps are requested before the first is stored (q is not known to
        // be distinct from w, so a store would otherwise wait for each load).
        const float *safe = in ? src : jb.w;
        float v[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) v[t] = safe[t < KS2 ? t : 0];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (t >= KS2) break;
            const int tq = jb.kind == 0 ? t : KS2 - 1 - t;
            jb.q[((int64_t)row * KS2 + tq) * jb.KP + col] = to_bf16(in ? v[t] : 0.f);
        }
    } else {
        const int e = (int)(i & 7), ln = (int)((i >> 3) & 63);
        const int64_t blk = i >> 9;
        const int ks = (int)(blk % jb.KP), mt = (int)(blk / jb.KP);
        const int row = mt * 32 + (ln & 31), col = ks * 16 + (ln >> 5) * 8 + e;
        float v = 0.f;
        if (jb.kind == 2) {
            if (row < CO && col < CI) v = jb.w[(int64_t)row * CI + col];
        } else {
            if (row < CI && col < CO) v = jb.w[(int64_t)col * CI + row];
        }
        jb.q[i] = to_bf16(v);
    }
}

}  // namespace rvn
