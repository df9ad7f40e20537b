// Row-wise 16-value codebook by 1-D k-means (Section 3, "Codebook-based Quantization"; Section 5:
// centres start on ASYM's uniform grid, codebooks are stored in binary16).
//
// One table row per lane, the row in registers (dimension a compile-time constant), the 16 centres
// in registers.  Per Lloyd round each element scans the 16 centres for the first nearest one
// (binary32 distances, strict '<', so equal distances keep the lower index) and adds its value to
// that cluster's binary64 sum; the sums and counts live in a lane-private column of LDS (16 KB per
// wave) because the cluster index is only known at run time (a register array cannot be indexed by
// it).  LDS operations of a wave execute in order, so a cluster's sum is accumulated in element
// order, which is what makes the result reproducible bit for bit.  Means are one binary64 division per
// non-empty cluster and round; empty clusters keep their centre.  After the fixed number of rounds
// the centres are rounded to binary16 and every element is assigned once more against the rounded
// codebook, so the stored indices and the stored codebook agree.
//
// Arithmetic per element and round, as the scan defines it: 16 subtractions, 8 three-input minimums,
// 15 compares, 15 selects and one binary64 add: about 55 operations; the path is bound by VALU issue
// like the greedy search.  With the centres in order (checked every round) the index comes from a
// bisection instead, 4 compares and 11 selects; with the centres well separated as well (the usual
// case), from a bisection over the centres that needs only the two distances to the bracketing centres.  Rows with dim <= 16 need no clustering (every value
// is its own codebook entry).
#pragma once

#include "greedy_rpl.h"  // load_row
#include "e4q_launch.h"

namespace e4q {

constexpr int kK = 16;
constexpr int kSeparatedBatch = 2;  // values whose nearest-centre bisections run side by side (4 and 8 measure the same)

// First index of the smallest |x - c[k]| (what a scan with a strict '<' finds).  Written as: the
// smallest distance (3-input minimum instructions), then the lowest index that attains it -- 16
// subtractions, 8 minimums, 15 compares and 15 selects instead of 15 compares and 30 selects.
__device__ __forceinline__ int nearest_centre(float x, const float (&c)[kK])
{
    float d[kK];
#pragma unroll
    for (int k = 0; k < kK; ++k) d[k] = __builtin_fabsf(x - c[k]);
    float m = __builtin_fminf(__builtin_fminf(d[0], d[1]), d[2]);
#pragma unroll
    for (int k = 3; k + 1 < kK; k += 2) m = __builtin_fminf(__builtin_fminf(m, d[k]), d[k + 1]);
    m = __builtin_fminf(m, d[kK - 1]);
    int idx = kK - 1;
#pragma unroll
    for (int k = kK - 2; k >= 0; --k) idx = (d[k] == m) ? k : idx;
    return idx;
}

// The same index when the centres are in non-decreasing order.  Then s[k] = x - c[k] (rounded) is
// non-increasing in k, "s[k] > m" (m the smallest distance) holds exactly for the centres before the
// first nearest one, and a four-step bisection over that predicate finds their number: 4 compares and
// 11 selects instead of 15 and 15.  The probe positions 7; 3|11; 1|5|9|13; 0|2|..|14 are picked by
// selects on the earlier outcomes, because a register array cannot be indexed at run time.
// UNIT scales the result (index * UNIT, UNIT a power of two), so that a caller that needs a byte offset
// gets it from the selects themselves.
template <int UNIT = 1>
__device__ __forceinline__ int nearest_centre_sorted(float x, const float (&c)[kK])
{
    float s[kK];
#pragma unroll
    for (int k = 0; k < kK; ++k) s[k] = x - c[k];
    float m = __builtin_fminf(__builtin_fminf(__builtin_fabsf(s[0]), __builtin_fabsf(s[1])), __builtin_fabsf(s[2]));
#pragma unroll
    for (int k = 3; k + 1 < kK; k += 2)
        m = __builtin_fminf(__builtin_fminf(m, __builtin_fabsf(s[k])), __builtin_fabsf(s[k + 1]));
    m = __builtin_fminf(m, __builtin_fabsf(s[kK - 1]));
    const bool b3 = s[7] > m;
    const float p2 = b3 ? s[11] : s[3];
    const bool b2 = p2 > m;
    const float u0 = b3 ? s[9] : s[1], u1 = b3 ? s[13] : s[5];
    const float p1 = b2 ? u1 : u0;
    const bool b1 = p1 > m;
    const float v0 = b3 ? s[8] : s[0], v1 = b3 ? s[10] : s[2], v2 = b3 ? s[12] : s[4], v3 = b3 ? s[14] : s[6];
    const float w0 = b2 ? v2 : v0, w1 = b2 ? v3 : v1;
    const float p0 = b1 ? w1 : w0;
    const bool b0 = p0 > m;
    return (b3 ? 8 * UNIT : 0) | (b2 ? 4 * UNIT : 0) | (b1 ? 2 * UNIT : 0) | (b0 ? UNIT : 0);
}

// The same index again, cheaper, when the centres are "well separated": strictly increasing with every
// gap c[k+1] - c[k] above 2^-22 of the row's range (centre_order below).  Then two different centres
// can never be at the same ROUNDED distance below a value x <= max: equal rounded differences
// x - c[a] == x - c[b] need |c[a] - c[b]| <= ulp(x - c) <= 2^-23 * range.  So the rounded distances to the
// centres at or below x strictly decrease towards x, those to the centres above x do not decrease,
// and the first nearest centre is one of the two that bracket x: the lower one unless the upper one
// is strictly nearer.  The bracket comes from a bisection over the centres themselves -- t = number
// of c[0..14] that are <= x -- which keeps the tighter probe on either side as it goes: 4 compares and
// 19 selects, then 2 subtractions and 1 compare, instead of 16 subtractions, 8 three-input minimums,
// 4 compares and 11 selects.  The result stays in 0..15 for any input, NaN included.
// N values are handled side by side, one bisection level at a time: a single value's chain (compare,
// select, compare, ...) is a dozen dependent instructions, which the two or three waves a SIMD holds
// cannot cover on their own.  (Measured on gfx950: a select on a condition in a scalar register pair
// issues every 4.4 cycles, like a compare; selects on VCC would issue every 2.4, but only if VCC was
// written some ten instructions earlier, and a wave has one VCC, so the conditions stay in register pairs.)
// `base` is added to the result (the caller's lane offset; base8 = base + 8 * UNIT), so that the first index
// bit brings it along and the sum of the five terms is two three-input additions.
template <int UNIT, int N>
__device__ __forceinline__ void nearest_centre_separated(const float (&x)[N], const float (&c)[kK], int base, int base8,
                                                         int (&out)[N])
{
    bool b3[N], b2[N], b1[N], b0[N];
    float below[N], above[N], p[N], u0[N], u1[N], v0[N], v1[N], v2[N], v3[N];
#pragma unroll
    for (int i = 0; i < N; ++i) b3[i] = x[i] >= c[7];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        below[i] = b3[i] ? c[7] : -__builtin_inff();
        above[i] = b3[i] ? c[15] : c[7];
        p[i] = b3[i] ? c[11] : c[3];
        u0[i] = b3[i] ? c[9] : c[1];
        u1[i] = b3[i] ? c[13] : c[5];
        v0[i] = b3[i] ? c[8] : c[0];
        v1[i] = b3[i] ? c[10] : c[2];
        v2[i] = b3[i] ? c[12] : c[4];
        v3[i] = b3[i] ? c[14] : c[6];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < N; ++i) b2[i] = x[i] >= p[i];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        below[i] = b2[i] ? p[i] : below[i];
        above[i] = b2[i] ? above[i] : p[i];
        p[i] = b2[i] ? u1[i] : u0[i];
        v0[i] = b2[i] ? v2[i] : v0[i];
        v1[i] = b2[i] ? v3[i] : v1[i];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < N; ++i) b1[i] = x[i] >= p[i];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        below[i] = b1[i] ? p[i] : below[i];
        above[i] = b1[i] ? above[i] : p[i];
        p[i] = b1[i] ? v1[i] : v0[i];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < N; ++i) b0[i] = x[i] >= p[i];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        below[i] = b0[i] ? p[i] : below[i];
        above[i] = b0[i] ? above[i] : p[i];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < N; ++i) {
        // no centre at or below x: below = -inf, the distance to it is +inf and the upper centre, c[0], wins
        const float dl = x[i] - below[i];
        const float du = __builtin_fabsf(x[i] - above[i]);
        out[i] = ((b3[i] ? base8 : base) + (b2[i] ? 4 * UNIT : 0) + (b1[i] ? 2 * UNIT : 0)) +
                 ((b0[i] ? UNIT : 0) + (dl <= du ? -UNIT : 0));
    }
}

template <int UNIT = 1>
__device__ __forceinline__ int nearest_centre_separated(float x, const float (&c)[kK])
{
    const float xs[1] = {x};
    int out[1];
    nearest_centre_separated<UNIT, 1>(xs, c, 0, 8 * UNIT, out);
    return out[0];
}

// Order of a row's centres: 2 = every gap c[k+1] - c[k] exceeds `min_gap` (well separated), 1 = non-decreasing,
// 0 = neither.  The smallest rounded gap decides all three (a rounded difference is negative exactly when the
// real one is).
__device__ __forceinline__ int centre_order(const float (&c)[kK], float min_gap)
{
    float g[kK - 1];
#pragma unroll
    for (int k = 0; k + 1 < kK; ++k) g[k] = c[k + 1] - c[k];
    float m = __builtin_fminf(__builtin_fminf(g[0], g[1]), g[2]);
#pragma unroll
    for (int k = 3; k + 1 < kK - 1; k += 2) m = __builtin_fminf(__builtin_fminf(m, g[k]), g[k + 1]);
    return m > min_gap ? 2 : (m >= 0.0f ? 1 : 0);
}

// The weakest order among the 64 rows of a wave (a NaN centre makes it 0).
__device__ __forceinline__ int wave_centre_order(const float (&c)[kK], float min_gap)
{
    const int o = centre_order(c, min_gap);
    if (__builtin_amdgcn_ballot_w64(o < 1) != 0) return 0;
    return __builtin_amdgcn_ballot_w64(o < 2) != 0 ? 1 : 2;
}

// True when every lane of the wave holds centres in non-decreasing order.  A grid is, and a Lloyd
// round keeps them so as long as every point goes to a centre of its own Voronoi cell; a point that
// ties between two centres through rounding goes to the lower index and can pull that centre past
// the other one.  No input is known to do that, but the order is checked every round rather than
// assumed, and a wave that fails the check scans all 16 centres (same results, more work).
__device__ __forceinline__ bool wave_centres_sorted(const float (&c)[kK])
{
    bool ok = true;
#pragma unroll
    for (int k = 0; k + 1 < kK; ++k) ok = ok && (c[k] <= c[k + 1]);
    return __builtin_amdgcn_ballot_w64(!ok) == 0;
}

__device__ __forceinline__ void grid_centres(float lo, float hi, float (&c)[kK])
{
    const float step = (hi - lo) / kQMax4;
#pragma unroll
    for (int k = 0; k < kK; ++k) c[k] = __builtin_fmaf((float)k, step, lo);
}

// Lane-private accumulators: slot k * 64 + l belongs to cluster k of lane l, so a wave's 64 slots of one
// access are consecutive in LDS and the binary64 accesses hit every bank evenly.  (Sum and count side by
// side in one 16-byte record was measured with bank conflicts in 47 % of the LDS cycles.)  12 KiB per wave:
// with 16 KiB (counts in 8-byte slots, which saved the shift in lloyd_add_at) a CU's 160 KiB of LDS held 10
// waves where the registers allow 12.
struct LloydScratch {
    double sum[kK * 64];
    uint32_t cnt[kK * 64];
};

__device__ __forceinline__ void lloyd_clear(LloydScratch& s, int lane)
{
#pragma unroll
    for (int k = 0; k < kK; ++k) {
        s.sum[k * 64 + lane] = 0.0;
        s.cnt[k * 64 + lane] = 0u;
    }
}

// The adds are LDS read-modify-write instructions without a return value (one instruction each
// instead of read, add, write): no other lane touches the slot, and a wave's LDS instructions
// execute in program order, so the sum still grows in element order.
__device__ __forceinline__ void lloyd_add(LloydScratch& s, int lane, int a, float x)
{
    const int slot = a * 64 + lane;
    __hip_atomic_fetch_add(&s.sum[slot], (double)x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    __hip_atomic_fetch_add(&s.cnt[slot], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

// Widening to binary64, pinned to where it is written.  The row's elements do not change between Lloyd
// rounds, so the compiler would otherwise widen each of them once before the first round and keep the
// results: two more registers per element for the whole kernel, which halves the number of waves a SIMD
// can hold (or worse) to save one conversion per element and round (measured at dimension 64: 3.83 ms
// with the widened copies kept, 2.80 ms without).
__device__ __forceinline__ double widen_here(float x)
{
    double d;
    asm volatile("v_cvt_f64_f32_e32 %0, %1" : "=v"(d) : "v"(x));
    return d;
}

// The same with the slot given as the byte offset of its sum, cluster * 512 + lane * 8; the count sits at
// half that offset in its own array.
__device__ __forceinline__ void lloyd_add_at(LloydScratch& s, int byte_offset, float x)
{
    double* sum = reinterpret_cast<double*>(reinterpret_cast<char*>(s.sum) + byte_offset);
    uint32_t* cnt = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(s.cnt) + (byte_offset >> 1));
    __hip_atomic_fetch_add(sum, widen_here(x), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

// The means of one round, GROUP clusters at a time: the group's LDS reads are all issued before its
// first division and the divisions carry no branch, so their dependent chains (about 15 binary64
// instructions each) interleave instead of running one after the other behind an LDS round trip
// each.  All 16 at once keeps 16 chains' temporaries alive on top of the row (more registers than
// two waves per SIMD leave); groups of 8 interleave as well and need half of that.
template <int GROUP = 8>
__device__ __forceinline__ void lloyd_update(const LloydScratch& s, int lane, float (&c)[kK])
{
#pragma unroll
    for (int g = 0; g < kK; g += GROUP) {
        uint32_t n[GROUP];
        double sum[GROUP];
#pragma unroll
        for (int k = 0; k < GROUP; ++k) {
            n[k] = s.cnt[(g + k) * 64 + lane];
            sum[k] = s.sum[(g + k) * 64 + lane];
        }
#pragma unroll
        for (int k = 0; k < GROUP; ++k) {
            float mean = (float)(sum[k] / (double)(n[k] > 0u ? n[k] : 1u));
            asm volatile("" : "+v"(mean));  // keeps the division out of a per-cluster branch
            c[g + k] = n[k] > 0u ? mean : c[g + k];
        }
        __builtin_amdgcn_sched_barrier(0);  // the next group's reads and divisions start after this group's
    }
}

// Writes the 16 centres of one row as binary16 (32 bytes).
__device__ __forceinline__ void store_codebook(const float (&c)[kK], uint16_t* __restrict__ cb)
{
    if (reinterpret_cast<uintptr_t>(cb) % 16 == 0) {
        uint32_t w[kK / 2];
#pragma unroll
        for (int k = 0; k < kK / 2; ++k)
            w[k] = (uint32_t)f16_bits(c[2 * k]) | ((uint32_t)f16_bits(c[2 * k + 1]) << 16);
        uint4* o = reinterpret_cast<uint4*>(cb);
        o[0] = make_uint4(w[0], w[1], w[2], w[3]);
        o[1] = make_uint4(w[4], w[5], w[6], w[7]);
    } else {
#pragma unroll
        for (int k = 0; k < kK; ++k) cb[k] = f16_bits(c[k]);
    }
}

// TAIL: the dimension d is not a multiple of 8 (D - 8 < d < D, the same for every lane).  Registers at
// and beyond d copy element 0 (min and max are unaffected), are skipped by scalar branches in the
// rounds and pack as index 0; a row of (d + 1) / 2 bytes is not a whole number of words, so the wave's
// 64 dense rows are assembled in LDS (in the accumulators' space, free by then) and copied out 16 bytes
// per lane at a time.
//
// WAVES: waves per workgroup, 1 or 4; they share nothing but the barrier of the TAIL path.  Tables of at most two
// waves per SIMD of the chip run in four-wave workgroups, whose waves land one on each SIMD of a compute unit, which
// one-wave workgroups do not (rows of 64 elements, one-wave -> four-wave workgroups: 65 536 rows 209 -> 153 us,
// 100 000 rows 284 -> 227 us, 131 072 rows 293 -> 233 us); from three waves per SIMD on, one-wave workgroups are 3 - 5 %
// faster (a compute unit's 160 KiB of LDS hold three four-wave workgroups, and a new one starts only when a whole one
// has ended).
template <int D, typename Tin, bool TAIL, int WAVES>
__device__ __forceinline__ void kmeans16_rpl_body(const KMeansArgs& a, int d, LloydScratch& scratch)
{
    static_assert(D > kK, "rows with dim <= 16 take the other kernel");
    const int lane = WAVES == 1 ? (int)threadIdx.x : (int)(threadIdx.x & 63u);
    const int64_t row0 = WAVES == 1 ? (int64_t)blockIdx.x * 64
                                    : ((int64_t)blockIdx.x * WAVES + (int64_t)(threadIdx.x >> 6)) * 64;
    const int64_t row = row0 + lane;
    const bool live = row < a.rows;
    const int64_t r = live ? row : a.rows - 1;
    const Tin* src = static_cast<const Tin*>(a.table) + r * a.row_stride;

    float x[D];
    if constexpr (TAIL) {
        float head[D - 8];
        load_row<D - 8>(src, a.vec_loads != 0, head);
#pragma unroll
        for (int k = 0; k < D - 8; ++k) x[k] = head[k];
#pragma unroll
        for (int k = D - 8; k < D; ++k) x[k] = (float)src[k < d ? k : 0];
    } else {
        load_row<D>(src, a.vec_loads != 0, x);
    }
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int k = 1; k < D; ++k) {
        lo = __builtin_fminf(lo, x[k]);
        hi = __builtin_fmaxf(hi, x[k]);
    }
    float c[kK];
    grid_centres(lo, hi, c);
    const float min_gap = (hi - lo) * 0x1p-22f;  // see nearest_centre_separated

    for (int it = 0; it < a.lloyd_iters; ++it) {
        lloyd_clear(scratch, lane);
        const int order = a.force_scan ? 0 : wave_centre_order(c, min_gap);  // uniform over the wave
        if (order == 2) {
            constexpr int N = kSeparatedBatch;
            static_assert(D % N == 0, "the batch divides the register row");
#pragma unroll
            for (int e = 0; e < D; e += N) {
                float xs[N];
                int slot[N];
#pragma unroll
                for (int i = 0; i < N; ++i) xs[i] = x[e + i];
                nearest_centre_separated<512, N>(xs, c, lane * 8, lane * 8 + 8 * 512, slot);
#pragma unroll
                for (int i = 0; i < N; ++i)  // element order, as the sums require
                    if (!TAIL || e + i < D - 7 || e + i < d) lloyd_add_at(scratch, slot[i], xs[i]);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if (order == 1) {
#pragma unroll
            for (int e = 0; e < D; ++e)
                if (!TAIL || e < D - 7 || e < d) lloyd_add_at(scratch, nearest_centre_sorted<512>(x[e], c) | (lane * 8), x[e]);
        } else {
            // rolled, re-reading the row: x[] cannot be indexed by a loop counter
#pragma unroll 1
            for (int e = 0; e < d; ++e) {
                const float v = (float)src[e];
                lloyd_add(scratch, lane, nearest_centre(v, c), v);
            }
        }
        lloyd_update(scratch, lane, c);
    }

    float ch[kK];
    constexpr int NWORDS = (D / 2 + 3) / 4;
    const int nbytes = (d + 1) / 2;
    uint32_t w[NWORDS];
#pragma unroll
    for (int k = 0; k < kK; ++k) ch[k] = through_f16(c[k]);
    const int final_order = a.force_scan ? 0 : wave_centre_order(ch, min_gap);
    if (final_order == 0) {
        if (live) {
            store_codebook(c, a.centroids_f16 + row * kK);
            uint8_t* out = a.idx + row * nbytes;
#pragma unroll 1
            for (int b = 0; b < nbytes; ++b) {
                const uint32_t q0 = (uint32_t)nearest_centre((float)src[2 * b], ch);
                const uint32_t q1 = (2 * b + 1 < d) ? (uint32_t)nearest_centre((float)src[2 * b + 1], ch) : 0u;
                out[b] = (uint8_t)(q0 | (q1 << 4));
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < NWORDS; ++i) {
        uint32_t acc = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (8 * i + e < D) {
                const uint32_t q = (uint32_t)(final_order == 2 ? nearest_centre_separated(x[8 * i + e], ch)
                                                               : nearest_centre_sorted(x[8 * i + e], ch));
                acc |= ((!TAIL || 8 * i + e < D - 7 || 8 * i + e < d) ? q : 0u) << (4 * e);
            }
        w[i] = acc;
    }
    if (live) store_codebook(c, a.centroids_f16 + row * kK);
    if constexpr (TAIL) {
        uint8_t* stage = reinterpret_cast<uint8_t*>(scratch.sum);  // 8 KiB; 64 rows of at most 64 bytes
        __syncthreads();
#pragma unroll
        for (int b = 0; b < D / 2; ++b)
            if (b < nbytes) stage[lane * nbytes + b] = (uint8_t)(w[b / 4] >> (8 * (b % 4)));
        __syncthreads();
        const int64_t rows_here = a.rows - row0 < 64 ? a.rows - row0 : 64;
        const int total = (int)rows_here * nbytes;
        uint8_t* dst = a.idx + row0 * nbytes;
        if (a.vec_stores == 2) {  // 16-byte aligned buffer: 64 * nbytes keeps every wave's start aligned
            for (int off = lane * 16; off < total; off += 64 * 16) {
                if (off + 16 <= total) {
                    *reinterpret_cast<uint4*>(dst + off) = *reinterpret_cast<const uint4*>(stage + off);
                } else {
                    for (int b = off; b < total; ++b) dst[b] = stage[b];
                }
            }
        } else {
            for (int b = lane; b < total; b += 64) dst[b] = stage[b];
        }
    } else {
        if (!live) return;
        uint8_t* out = a.idx + row * (D / 2);
        if (a.vec_stores >= 1) {
            uint32_t* o = reinterpret_cast<uint32_t*>(out);
#pragma unroll
            for (int i = 0; i < NWORDS; ++i) o[i] = w[i];
        } else {
#pragma unroll
            for (int b = 0; b < D / 2; ++b) out[b] = (uint8_t)(w[b / 4] >> (8 * (b % 4)));
        }
    }
}

template <int D, typename Tin, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) kmeans16_rpl_kernel(KMeansArgs a)
{
    __shared__ LloydScratch scratch[WAVES];
    kmeans16_rpl_body<D, Tin, false, WAVES>(a, D, scratch[WAVES == 1 ? 0 : threadIdx.x >> 6]);
}

template <int D, typename Tin, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) kmeans16_rpl_tail_kernel(KMeansArgs a, int32_t d)
{
    __shared__ LloydScratch scratch[WAVES];
    kmeans16_rpl_body<D, Tin, true, WAVES>(a, d, scratch[WAVES == 1 ? 0 : threadIdx.x >> 6]);
}

// Waves per workgroup for a table of `rows` rows of (rounded-up) dimension D (see kmeans16_rpl_body): four while the
// launch has at most one wave per SIMD less than the registers let a SIMD hold (three waves up to D = 88, two
// beyond).  Measured, one-wave -> four-wave workgroups: D = 128, 65 536 rows 373 -> 276 us, 131 072 rows 402 -> 421 us;
// D = 32, 131 072 rows 174 -> 141 us, 200 000 rows 239 -> 239 us.
inline int kmeans16_waves_per_block(const KMeansArgs& a, int D)
{
    if (a.waves == 1 || a.waves == 4) return (int)a.waves;
    const int64_t resident = D <= 88 ? 3 : 2;
    return a.rows <= (resident - 1) * (int64_t)1024 * 64 ? 4 : 1;
}

// Launches the register-resident kernel for `dim` if there is one; returns false otherwise.
template <typename Tin>
inline bool launch_kmeans16_rpl(const KMeansArgs& a, int32_t dim, hipStream_t stream)
{
    const int waves = kmeans16_waves_per_block(a, dim);
    const dim3 grid((unsigned)((a.rows + 64 * waves - 1) / (64 * waves))), block(64 * waves);
    switch (dim) {
#define E4Q_CASE(D) \
    case D:         \
        if (waves == 1) hipLaunchKernelGGL((kmeans16_rpl_kernel<D, Tin, 1>), grid, block, 0, stream, a); \
        else hipLaunchKernelGGL((kmeans16_rpl_kernel<D, Tin, 4>), grid, block, 0, stream, a);           \
        return true;
        E4Q_CASE(24) E4Q_CASE(32) E4Q_CASE(40) E4Q_CASE(48) E4Q_CASE(56) E4Q_CASE(64) E4Q_CASE(72)
        E4Q_CASE(80) E4Q_CASE(88) E4Q_CASE(96) E4Q_CASE(104) E4Q_CASE(112) E4Q_CASE(120) E4Q_CASE(128)
#undef E4Q_CASE
        default:
            return false;
    }
}

// The same for 16 < dim < 128, dim % 8 != 0: the kernel of the next multiple of 8 with a masked tail.
template <typename Tin>
inline bool launch_kmeans16_rpl_tail(const KMeansArgs& a, int32_t dim, hipStream_t stream)
{
    if (dim <= kK || dim >= 128 || dim % 8 == 0) return false;
    const int waves = kmeans16_waves_per_block(a, (dim + 7) / 8 * 8);
    const dim3 grid((unsigned)((a.rows + 64 * waves - 1) / (64 * waves))), block(64 * waves);
    switch ((dim + 7) / 8 * 8) {
#define E4Q_CASE(D) \
    case D:         \
        if (waves == 1) hipLaunchKernelGGL((kmeans16_rpl_tail_kernel<D, Tin, 1>), grid, block, 0, stream, a, dim); \
        else hipLaunchKernelGGL((kmeans16_rpl_tail_kernel<D, Tin, 4>), grid, block, 0, stream, a, dim);           \
        return true;
        E4Q_CASE(24) E4Q_CASE(32) E4Q_CASE(40) E4Q_CASE(48) E4Q_CASE(56) E4Q_CASE(64) E4Q_CASE(72)
        E4Q_CASE(80) E4Q_CASE(88) E4Q_CASE(96) E4Q_CASE(104) E4Q_CASE(112) E4Q_CASE(120) E4Q_CASE(128)
#undef E4Q_CASE
        default:
            return false;
    }
}

}  // namespace e4q
