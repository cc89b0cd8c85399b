// Row arithmetic shared by the softmax kernels: wavefront / workgroup reductions
// and the exponential.  Internal, device only.
#pragma once

#include "common.hpp"

namespace cnnmem {

// ---- wavefront reductions ----------------------------------------------------
// DPP controls: quad_perm(1,0,3,2)=0xB1, quad_perm(2,3,0,1)=0x4E,
// row_half_mirror=0x141, row_mirror=0x140.  After the four steps every lane of a
// 16-lane row holds the row's result; the four rows are combined by reading one
// lane of each.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}

__device__ __forceinline__ float lane_value(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

struct MaxOp {
    static __device__ __forceinline__ float apply(float a, float b) { return fmaxf(a, b); }
};
struct SumOp {
    static __device__ __forceinline__ float apply(float a, float b) { return a + b; }
};

template <class Op>
__device__ __forceinline__ float wave_reduce(float v) {
    v = Op::apply(v, dpp_move<0xB1>(v));
    v = Op::apply(v, dpp_move<0x4E>(v));
    v = Op::apply(v, dpp_move<0x141>(v));
    v = Op::apply(v, dpp_move<0x140>(v));
    const float r0 = lane_value(v, 0), r1 = lane_value(v, 16);
    const float r2 = lane_value(v, 32), r3 = lane_value(v, 48);
    return Op::apply(Op::apply(r0, r1), Op::apply(r2, r3));
}

// Reduction over the TPR lanes that share a row.  `slots` has one float per
// wavefront of the workgroup; `first_wave` is the row's first wavefront.  FRESH: nothing has used `slots`
// before in this kernel (each reduction has an array of its own), which saves the barrier that otherwise
// separates this use from the previous one: two barriers per row instead of four.
template <class Op, int TPR, bool FRESH = false>
__device__ __forceinline__ float row_reduce(float v, float* slots, int wave, int first_wave) {
    v = wave_reduce<Op>(v);
    if constexpr (TPR > kWave) {
        constexpr int WAVES = TPR / kWave;
        if constexpr (!FRESH) __syncthreads();      // previous use of slots is over
        if ((threadIdx.x & (kWave - 1)) == 0) slots[wave] = v;
        __syncthreads();
        float r = slots[first_wave];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) r = Op::apply(r, slots[first_wave + w]);
        v = r;
    }
    return v;
}

// Reduction over a group of G = 4 .. 32 neighbouring lanes (G a power of two, groups aligned
// to G): every lane of the group ends up with the group's result.  All 64 lanes of the
// wavefront must take part.
template <class Op, int G>
__device__ __forceinline__ float group_reduce(float v) {
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) v = Op::apply(v, __shfl_xor(v, off, G));
    return v;
}

// exp(d) for d <= 0, about 1 ulp: 2^t with t = d*log2(e) rounded once, then a
// first-order correction for the rounding error of that product.  Arguments
// below -120 give exactly 0 (they are below the smallest fp32 denormal anyway).
__device__ __forceinline__ float exp_nonpos(float d) {
    constexpr float kLog2eHi = 1.44269502162933349609375f;        // fp32(log2 e)
    constexpr float kLog2eLo = 1.925963033500011e-08f;            // log2 e - fp32(log2 e)
    constexpr float kLn2 = 0.693147182464599609375f;
    d = fmaxf(d, -120.0f);
    const float t = d * kLog2eHi;
    float err = __builtin_fmaf(d, kLog2eHi, -t);                  // exact product minus its rounding
    err = __builtin_fmaf(d, kLog2eLo, err);
    const float p = __builtin_amdgcn_exp2f(t);
    return __builtin_fmaf(p, err * kLn2, p);
}

constexpr float kRowNegInf = -__builtin_huge_valf();


}  // namespace cnnmem
