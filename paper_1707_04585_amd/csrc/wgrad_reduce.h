// Ordered sum of the filter-gradient partial results, shared by the kernels
// that can carry it: dw (+)= sum_s part[s], with the slot mapped from the
// matrix instruction's register order to dw[ko][c][tap].  Device code only.
#pragma once

#include "kernels.h"

namespace rvn {

// One workgroup of 256 threads handles 32 consecutive partial-result slots: 8
// slices of s are summed in order by 8 groups of 32 threads, then combined in
// order.  `lds` holds 256 floats.  `block` counts from 0 to r.blocks - 1.
// With few slices (r.wide) a thread owns one slot and sums all S slices itself,
// 256 slots per workgroup.
__device__ __forceinline__ void wgrad_reduce_body(const WgradReduce &r, int block, float *lds) {
    int o;
    float t = 0.f;
    bool mine;
    if (r.wide) {
        o = block * 256 + threadIdx.x;
        mine = o < r.part_stride;
        if (mine) {
            const float *q = r.part + o;
            int s = 0;
            for (; s + 4 <= r.S; s += 4) {
                const float a = q[(int64_t)s * r.part_stride], b = q[(int64_t)(s + 1) * r.part_stride];
                const float c = q[(int64_t)(s + 2) * r.part_stride], d = q[(int64_t)(s + 3) * r.part_stride];
                t += (a + b) + (c + d);
            }
            for (; s < r.S; ++s) t += q[(int64_t)s * r.part_stride];
        }
    } else {
        o = block * 32 + (threadIdx.x & 31);
        const int sl = threadIdx.x >> 5;
        const int per = (r.S + 7) / 8;
        const int s0 = sl * per, s1 = min(r.S, s0 + per);
        float v = 0.f;
        if (o < r.part_stride) {
            const float *q = r.part + o;
            int s = s0;
            for (; s + 4 <= s1; s += 4) {
                const float a = q[(int64_t)s * r.part_stride], b = q[(int64_t)(s + 1) * r.part_stride];
                const float c = q[(int64_t)(s + 2) * r.part_stride], d = q[(int64_t)(s + 3) * r.part_stride];
                v += (a + b) + (c + d);
            }
            for (; s < s1; ++s) v += q[(int64_t)s * r.part_stride];
        }
        lds[threadIdx.x] = v;
        __syncthreads();
        mine = sl == 0 && o < r.part_stride;
        if (mine) {
            const int l = threadIdx.x;
            t = ((lds[l] + lds[32 + l]) + (lds[64 + l] + lds[96 + l])) +
                ((lds[128 + l] + lds[160 + l]) + (lds[192 + l] + lds[224 + l]));
        }
    }
    if (mine) {
        const int WT = r.MT * r.CT;
        const int ln = o & 63;
        int ko_in, c_in, rest;
        if (r.tile == 16) {  // v_mfma_f32_16x16x4_f32: 4 registers per lane
            const int j = (o >> 6) & 3;
            rest = o >> 8;
            ko_in = 4 * (ln >> 4) + j;
            c_in = ln & 15;
        } else {  // v_mfma_f32_32x32x16_bf16: 16 registers per lane
            const int i = (o >> 6) & 15;
            rest = o >> 10;
            ko_in = 8 * (i >> 2) + 4 * (ln >> 5) + (i & 3);
            c_in = ln & 31;
        }
        const int tap = rest % r.KS2;
        rest /= r.KS2;
        const int tl = rest % WT, grp = rest / WT;
        const int gy = grp / r.tiles_c, gz = grp - gy * r.tiles_c;
        const int mm = tl / r.CT, cc = tl - mm * r.CT;
        const int ko = (gy * r.MT + mm) * r.tile + ko_in, c = (gz * r.CT + cc) * r.tile + c_in;
        if (ko < r.CO && c < r.CI) {
            const int64_t i = ((int64_t)ko * r.CI + c) * r.KS2 + tap;
            r.dw[i] = r.accumulate ? r.dw[i] + t : t;
        }
    }
}

}  // namespace rvn
