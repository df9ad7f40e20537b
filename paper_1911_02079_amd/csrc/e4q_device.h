// Device-side building blocks shared by the quantization kernels (gfx950, wave64).
//
// Arithmetic contract (this is what makes results reproducible bit for bit):
//   * everything is IEEE binary32, round-to-nearest-even, one rounding per written operation;
//     the translation units are compiled with -ffp-contract=off so that the compiler fuses
//     nothing on its own, and the one fused operation (the dequantizer scale*q+bias) is written
//     as an explicit fma;
//   * divisions are correctly rounded (-fhip-fp32-correctly-rounded-divide-sqrt);
//   * a row's squared errors are added by a balanced tree over index-adjacent pairs
//     (zero padded to a power of two; adding +0 is the identity on the non-negative terms, so
//     padded leaves are simply left out).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace e4q {

constexpr float kQMax = 15.0f;  // 2^n - 1 for n = 4 (Eq. 1)

// Value after a round trip through binary16 (RNE; v_cvt_f16_f32 then v_cvt_f32_f16).
__device__ __forceinline__ float through_f16(float v) { return (float)(_Float16)v; }

__device__ __forceinline__ uint16_t f16_bits(float v)
{
    _Float16 h = (_Float16)v;
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float f16_bits_to_float(uint16_t b)
{
    return (float)__builtin_bit_cast(_Float16, b);
}

// The parameters that are stored for the clipping range [lo, hi] (Eq. 1 with binary16 storage):
// scale = (hi - lo)/15 and bias = lo, both rounded to binary16, and the reciprocal used by the
// quantizer (0 when the range collapses, which sends every code to 0).
struct StoredParams {
    float scale, bias, inv;
};

__device__ __forceinline__ StoredParams stored_params(float lo, float hi)
{
    StoredParams p;
    float scale32 = (hi - lo) / kQMax;
    p.scale = through_f16(scale32);
    p.bias = through_f16(lo);
    p.inv = (p.scale == 0.0f) ? 0.0f : 1.0f / p.scale;
    return p;
}

// x_int of Eq. 1 as a float in {0..15}: round-half-even of (x - bias) * (1/scale), clamped.
__device__ __forceinline__ float quantize_elem(float x, const StoredParams& p)
{
    float t = (x - p.bias) * p.inv;
    return __builtin_amdgcn_fmed3f(__builtin_rintf(t), 0.0f, kQMax);
}

// Squared reconstruction error of one element (one term of Eq. 2): 8 VALU operations.
__device__ __forceinline__ float elem_sq_err(float x, const StoredParams& p)
{
    float q = quantize_elem(x, p);
    float xh = __builtin_fmaf(q, p.scale, p.bias);
    float e = x - xh;
    return e * e;
}

// Balanced adjacent-pair sum of leaf(LO) .. leaf(min(LO+SPAN, D)-1); SPAN is a power of two.
// `leaf` is called with a compile-time index (std::integral_constant style) so that rows held in
// registers stay in registers.
template <int K>
struct Idx {
    static constexpr int value = K;
};

template <int LO, int SPAN, int D, class Leaf>
__device__ __forceinline__ float tree_sum(Leaf&& leaf)
{
    static_assert(LO < D, "empty subtree");
    if constexpr (SPAN == 1) {
        return leaf(Idx<LO>{});
    } else {
        constexpr int H = SPAN / 2;
        if constexpr (LO + H >= D) {
            return tree_sum<LO, H, D>(leaf);  // right half is padding
        } else {
            float a = tree_sum<LO, H, D>(leaf);
            float b = tree_sum<LO + H, H, D>(leaf);
            return a + b;
        }
    }
}

constexpr int next_pow2(int d)
{
    int p = 1;
    while (p < d) p *= 2;
    return p;
}

}  // namespace e4q
