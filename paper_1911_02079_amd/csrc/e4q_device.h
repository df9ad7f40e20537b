// Device-side building blocks shared by the quantization kernels (gfx950, wave64).
//
// Arithmetic contract (this is what makes results reproducible bit for bit):
//   * everything is IEEE binary32, round-to-nearest-even, one rounding per written operation;
//     the translation units are compiled with -ffp-contract=off so that the compiler fuses
//     nothing on its own, and the one fused operation (the dequantizer scale*q+bias) is written
//     as an explicit fma;
//   * divisions are correctly rounded (-fhip-fp32-correctly-rounded-divide-sqrt; the two per scored range
//     by a shorter sequence with the same results, see div_by_qmax);
//   * a row's squared errors are added by a balanced tree over index-adjacent pairs
//     (zero padded to a power of two; adding +0 is the identity on the non-negative terms, so
//     padded leaves are simply left out).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <utility>

namespace e4q {

constexpr float kQMax4 = 15.0f;  // 2^n - 1 for n = 4 (Eq. 1); the codebook grid uses it directly

// Value after a round trip through binary16 (RNE; v_cvt_f16_f32 then v_cvt_f32_f16).
// Hides where a binary32 value came from.  Without it the compiler folds the widening of a binary16
// value into every multiply-add that uses it (the mixed-precision form of the instruction), which
// issues at a fraction of the plain binary32 rate; the result is the same either way.
__device__ __forceinline__ float opaque(float v)
{
    asm("" : "+v"(v));
    return v;
}

// Rounding to binary16 always starts from a finished binary32 value: the input is hidden as well, so that
// the conversion cannot be merged with the operation that produced it into one mixed-precision
// instruction with a single rounding (seen with a multiply-add as producer).
__device__ __forceinline__ float through_f16(float v) { return opaque((float)(_Float16)opaque(v)); }

__device__ __forceinline__ uint16_t f16_bits(float v)
{
    _Float16 h = (_Float16)opaque(v);
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float f16_bits_to_float(uint16_t b)
{
    return opaque((float)__builtin_bit_cast(_Float16, b));
}

// -0 becomes +0, every other value stays (round-to-nearest: -0 + +0 = +0).
__device__ __forceinline__ float canonical_zero(float v) { return v + 0.0f; }

// The parameters that are stored for the clipping range [lo, hi] (Eq. 1 with binary16 storage):
// scale = (hi - lo)/(2^n - 1) and bias = lo, both rounded to binary16, the reciprocal used by the
// quantizer (0 when the range collapses, which sends every code to 0), and the largest code.
struct StoredParams {
    float scale, bias, inv, qmax;
};

// The two divisions behind every scored range, in three instructions each instead of the thirteen of the
// general division sequence (at dimension 8 the general sequences are a fifth of the search; at 128, 2 %).
//   x / qmax:  q = x * rq with rq = 1/qmax rounded, then one correction by the exact remainder x - qmax * q.
//   1 / s:     the hardware reciprocal and one Newton step.
// Both return the correctly rounded IEEE quotient for every argument the search can produce: checked on
// the device against the division sequence over all 2^32 binary32 x for qmax = 3, 15 and 255 (equal for every
// finite x except -0, where the result is +0; a range hi - lo is never -0) and over all 65 536 binary16 s
// (csrc/probes/division_check.hip).
__device__ __forceinline__ float div_by_qmax(float x, float qmax, float rq)
{
    const float q = x * rq;
    const float r = __builtin_fmaf(-qmax, q, x);
    return __builtin_fmaf(r, rq, q);
}

// s: a value representable in binary16, not 0.
__device__ __forceinline__ float rcp_of_f16_value(float s)
{
    const float y = __builtin_amdgcn_rcpf(s);
    const float e = __builtin_fmaf(-s, y, 1.0f);
    return __builtin_fmaf(e, y, y);
}

__device__ __forceinline__ StoredParams stored_params(float lo, float hi, float qmax)
{
    StoredParams p;
    const float rq = 1.0f / qmax;  // the same for every range of the kernel: computed once
    p.scale = through_f16(div_by_qmax(hi - lo, qmax, rq));
    p.bias = through_f16(lo);
    const float inv = rcp_of_f16_value(p.scale);
    p.inv = (p.scale == 0.0f) ? 0.0f : inv;
    p.qmax = qmax;
    return p;
}

// The same parameters rebuilt from what is stored (the final encode uses exactly the stored bits).
__device__ __forceinline__ StoredParams params_from_bits(uint16_t scale_bits, uint16_t bias_bits, float qmax)
{
    StoredParams p;
    p.scale = f16_bits_to_float(scale_bits);
    p.bias = f16_bits_to_float(bias_bits);
    p.inv = (p.scale == 0.0f) ? 0.0f : 1.0f / p.scale;
    p.qmax = qmax;
    return p;
}

// x_int of Eq. 1 as a float in {0..qmax}: round-half-even of (x - bias) * (1/scale), clamped.
__device__ __forceinline__ float quantize_elem(float x, const StoredParams& p)
{
    float t = (x - p.bias) * p.inv;
    return __builtin_amdgcn_fmed3f(__builtin_rintf(t), 0.0f, p.qmax);
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

// Eq. 2 restricted to elements LO .. LO+SPAN-1 (those below D) of a row held in registers, summed
// over the same adjacent-pair tree as tree_sum.  MASKED drops elements at or beyond `nvalid`;
// elements below VALID_BELOW are known to exist and carry no test.
// Per element: quantize_elem's three steps, then xh = fma(q, scale, bias), e = x - xh, e * e.
//
// Below kStage elements the arithmetic runs one step at a time over the whole block with the
// instruction order pinned, instead of element by element: the compiler's own order keeps two
// elements in flight, too few to cover the result latency with three waves on a SIMD.  On gfx950 a
// wave64 binary32 add, multiply or multiply-add occupies the SIMD for 2 clocks, while rounding and
// the three-operand clamp take 4; the wave lowers its priority for the run of those two steps and
// raises it again afterwards, so that waves in their cheap steps are issued first and the others
// fill in (measured 4 % to 12 % over no hint; priorities inside a kernel only order waves of a SIMD).
constexpr int kStage = 4;

// The mask of tree_sq_err when `nvalid` is the same for every lane (UNIFORM_MASK): a multiplication by 1.0f or
// 0.0f held in a scalar register the optimizer cannot see through (a squared error is finite and not
// negative, so the product is the term itself or +0.0f, what a select would give): a select on a
// wave-uniform condition is turned into a branch around the element's arithmetic, and with a branch
// in the block the rest of the arithmetic is moved behind it, out of the pinned order.
__device__ __forceinline__ float uniform_keep_factor(bool exists)
{
    uint32_t m = exists ? 0x3f800000u : 0u;  // the bits of 1.0f or 0.0f, selected on the scalar unit
    asm volatile("" : "+s"(m));
    return __builtin_bit_cast(float, m);
}

// With a mask that differs between lanes (MASKED without UNIFORM_MASK) the caller passes `keep`, one factor per
// element, 1.0f where the element exists and 0.0f where it does not, made once per row and hidden from the
// optimizer in the same way (lane_keep_factor); otherwise `keep` is not read.
__device__ __forceinline__ float lane_keep_factor(bool exists)
{
    float m = exists ? 1.0f : 0.0f;
    asm("" : "+v"(m));
    return m;
}

template <int LO, int SPAN, int D, bool MASKED, int VALID_BELOW = 0, bool UNIFORM_MASK = false>
__device__ __forceinline__ float tree_sq_err(const float (&x)[D], const StoredParams& p, int nvalid,
                                             const float (&keep)[D])
{
    static_assert(LO < D, "empty subtree");
    if constexpr (SPAN <= kStage) {
        constexpr int N = (D - LO) < SPAN ? (D - LO) : SPAN;
        float t[N];
#pragma unroll
        for (int i = 0; i < N; ++i) t[i] = x[LO + i] - p.bias;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < N; ++i) t[i] = t[i] * p.inv;
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
#pragma unroll
        for (int i = 0; i < N; ++i) t[i] = __builtin_rintf(t[i]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < N; ++i) t[i] = __builtin_amdgcn_fmed3f(t[i], 0.0f, p.qmax);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int i = 0; i < N; ++i) t[i] = __builtin_fmaf(t[i], p.scale, p.bias);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < N; ++i) t[i] = x[LO + i] - t[i];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < N; ++i) t[i] = t[i] * t[i];
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (MASKED) {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                if (LO + i < VALID_BELOW) continue;
                if constexpr (UNIFORM_MASK) t[i] = t[i] * uniform_keep_factor(LO + i < nvalid);
                else t[i] = t[i] * keep[LO + i];
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        const float s = tree_sum<0, SPAN, N>([&](auto k) { return t[decltype(k)::value]; });
        __builtin_amdgcn_sched_barrier(0);
        return s;
    } else {
        constexpr int H = SPAN / 2;
        if constexpr (LO + H >= D) {
            return tree_sq_err<LO, H, D, MASKED, VALID_BELOW, UNIFORM_MASK>(x, p, nvalid, keep);  // right half is padding
        } else {
            const float a = tree_sq_err<LO, H, D, MASKED, VALID_BELOW, UNIFORM_MASK>(x, p, nvalid, keep);
            const float b = tree_sq_err<LO + H, H, D, MASKED, VALID_BELOW, UNIFORM_MASK>(x, p, nvalid, keep);
            return a + b;
        }
    }
}

// Packs N codes of NBITS bits (8/NBITS per byte, first element in the lowest bits) into 32-bit words.
// `code(Idx<k>)` returns element k's code as an unsigned integer (0 for elements that do not exist).
template <int NBITS, class Code, int... K>
__device__ __forceinline__ void pack_codes_impl(Code& code, uint32_t* w, std::integer_sequence<int, K...>)
{
    constexpr int PER_WORD = 32 / NBITS;
    ((w[K / PER_WORD] |= (uint32_t)code(Idx<K>{}) << ((K % PER_WORD) * NBITS)), ...);
}

template <int NBITS, int N, class Code>
__device__ __forceinline__ void pack_codes(Code&& code, uint32_t (&w)[(N * NBITS + 31) / 32])
{
    constexpr int NWORDS = (N * NBITS + 31) / 32;
#pragma unroll
    for (int i = 0; i < NWORDS; ++i) w[i] = 0;
    pack_codes_impl<NBITS>(code, w, std::make_integer_sequence<int, N>{});
}

// Stores the first `nbytes_live` of NBYTES packed bytes held in w[] at `out`: 16-byte or 4-byte
// stores when the row size and the alignment class of the buffer allow it, single bytes otherwise.
// `align_class`: 0 = unknown, 1 = `out` is 4-byte aligned, 2 = 16-byte aligned.
template <int NBYTES>
__device__ __forceinline__ void store_packed(uint8_t* __restrict__ out, const uint32_t (&w)[(NBYTES + 3) / 4],
                                             uint32_t align_class, int nbytes_live = NBYTES)
{
    constexpr int NWORDS = (NBYTES + 3) / 4;
    if (NBYTES % 16 == 0 && align_class == 2 && nbytes_live == NBYTES) {
        uint4* o4 = reinterpret_cast<uint4*>(out);
#pragma unroll
        for (int i = 0; i + 3 < NWORDS; i += 4) o4[i / 4] = make_uint4(w[i], w[i + 1], w[i + 2], w[i + 3]);
    } else if (NBYTES % 4 == 0 && align_class >= 1 && nbytes_live % 4 == 0) {
        uint32_t* o1 = reinterpret_cast<uint32_t*>(out);
#pragma unroll
        for (int i = 0; i < NWORDS; ++i)
            if (4 * i < nbytes_live) o1[i] = w[i];
    } else {
#pragma unroll
        for (int b = 0; b < NBYTES; ++b)
            if (b < nbytes_live) out[b] = (uint8_t)(w[b / 4] >> (8 * (b % 4)));
    }
}

// Quantizes, packs and stores the codes of x[C0 .. N), 16 bytes of codes at a time: a chunk is
// finished before the next one starts, so the encode needs few registers beyond x itself.  N is a
// multiple of 8.  With MASKED only the first `nvalid` elements exist: the others pack as 0 and bytes
// that hold no existing element are not written.
template <int NB, int N, int C0, bool MASKED>
__device__ __forceinline__ void encode_chunks(const float (&x)[N], const StoredParams& p, int nvalid,
                                              uint8_t* __restrict__ out, uint32_t align_class, bool live)
{
    if constexpr (C0 < N) {
        constexpr int CH = 128 / NB;                         // elements in 16 bytes of codes
        constexpr int M = (N - C0 < CH) ? N - C0 : CH;       // elements in this chunk
        constexpr int CHUNK_BYTES = M * NB / 8;
        uint32_t w[(M * NB + 31) / 32];
        pack_codes<NB, M>([&](auto k) {
            constexpr int e = C0 + decltype(k)::value;
            const uint32_t q = (uint32_t)quantize_elem(x[e], p);
            return (!MASKED || e < nvalid) ? q : 0u;
        }, w);
        int live_bytes = CHUNK_BYTES;
        if constexpr (MASKED) live_bytes = min(max((nvalid * NB + 7) / 8 - C0 * NB / 8, 0), CHUNK_BYTES);
        if (live) store_packed<CHUNK_BYTES>(out + C0 * NB / 8, w, align_class, live_bytes);
        encode_chunks<NB, N, C0 + CH, MASKED>(x, p, nvalid, out, align_class, live);
    }
}

constexpr int next_pow2(int d)
{
    int p = 1;
    while (p < d) p *= 2;
    return p;
}

}  // namespace e4q
