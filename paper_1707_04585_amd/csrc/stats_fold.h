// The fold used by convolution epilogues that leave statistics of their output
// for the next BN layer: a wavefront half (32 lanes) holds 16 channels per lane,
// each lane a sum over its own pixels; four steps halve the channels a lane
// holds and add the partner lane's, a fifth adds the last pair.  Afterwards
// lane l of the half holds the total of register l / 2 (both lanes of a pair
// hold the same).  Every sum has a fixed order.  Device code only.
#pragma once

namespace rvn {

namespace {

// One step: a lane holding CNT channels keeps the lower or upper half (by bit
// CNT of its index in the half) and adds the same half of the lane CNT away;
// the pivot of a kept channel moves along.
template <int CNT>
__device__ __forceinline__ void fold_step(float (&ea)[16], float (&eb)[16], float (&piv)[16], int l32) {
    constexpr int H = CNT / 2;
    const bool up = (l32 & CNT) != 0;
#pragma unroll
    for (int k = 0; k < H; ++k) {
        const float keep_a = up ? ea[k + H] : ea[k], send_a = up ? ea[k] : ea[k + H];
        const float keep_b = up ? eb[k + H] : eb[k], send_b = up ? eb[k] : eb[k + H];
        ea[k] = keep_a + __shfl_xor(send_a, CNT, 64);
        eb[k] = keep_b + __shfl_xor(send_b, CNT, 64);
        piv[k] = up ? piv[k + H] : piv[k];
    }
}

// ea, eb: per register the lane's sums of (v - pivot) and (v - pivot)^2; piv: the
// pivots (uniform over the half).  On return element 0 of each belongs to
// register l32 / 2.
__device__ __forceinline__ void fold_16_channels(float (&ea)[16], float (&eb)[16], float (&piv)[16], int l32) {
    fold_step<16>(ea, eb, piv, l32);
    fold_step<8>(ea, eb, piv, l32);
    fold_step<4>(ea, eb, piv, l32);
    fold_step<2>(ea, eb, piv, l32);
    ea[0] += __shfl_xor(ea[0], 1, 64);
    eb[0] += __shfl_xor(eb[0], 1, 64);
}

}  // namespace

}  // namespace rvn
