// Greedy clip search, one table row per LANE ("row-per-lane").
//
// Each lane of a wave owns one row and keeps its D elements in D vector registers for the whole
// search (Algorithm 1 scores 1 + 2*n_iter ranges per row, 65 at the paper's defaults, so the row
// is read from HBM once and reused from registers).  Because a lane owns a whole row there is no
// cross-lane traffic at all: min/max, the per-range scale/bias/reciprocal, the error sum and the
// greedy decisions are all lane-local, and every lane does useful work in every instruction.
// The loop trip count is the same for every row, so the wave never diverges.
//
// The waves of a workgroup share nothing.  A table of fewer than 8 waves per SIMD runs in four-wave workgroups, whose
// waves are spread over the four SIMDs of a compute unit, which one-wave workgroups are not (measured: with one to
// two waves per SIMD on average, or exactly four, tables of 100 000 - 260 000 rows ran 15 - 50 % longer in one-wave
// workgroups); larger tables run in one-wave workgroups (the same speed within 0.5 %, a batch of 26 tables 1.5 % faster).
// The kernels take the workgroup size from the launch.
//
// Memory access: lane l reads row (base + l) in 16-byte pieces; across the wave these are 64
// different cache lines per instruction, which costs a few thousand cycles per wave once, against
// some 150 000 cycles of arithmetic for D = 128 -- the kernel is bound by VALU issue, not by HBM.
// Codes go out as 16-byte (or 4-byte) stores per lane into the dense code array, scale and bias
// as one 2-byte store per lane (128 contiguous bytes per wave).
#pragma once

#include "e4q_device.h"
#include "e4q_launch.h"

namespace e4q {

constexpr int kRplBlock = kRplMaxRowsPerBlock;  // largest workgroup: four independent waves; no LDS, no barriers

template <int D>
__device__ __forceinline__ void load_row(const float* __restrict__ row, bool vec, float (&x)[D])
{
    if constexpr (D % 4 == 0) {
        if (vec) {
            const float4* r4 = reinterpret_cast<const float4*>(row);
#pragma unroll
            for (int k = 0; k < D / 4; ++k) {
                float4 v = r4[k];
                x[4 * k + 0] = v.x;
                x[4 * k + 1] = v.y;
                x[4 * k + 2] = v.z;
                x[4 * k + 3] = v.w;
            }
            return;
        }
    }
#pragma unroll
    for (int k = 0; k < D; ++k) x[k] = row[k];
}

template <int D>
__device__ __forceinline__ void load_row(const _Float16* __restrict__ row, bool vec, float (&x)[D])
{
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    if constexpr (D % 8 == 0) {
        if (vec) {
            const half8* r8 = reinterpret_cast<const half8*>(row);
#pragma unroll
            for (int k = 0; k < D / 8; ++k) {
                half8 v = r8[k];
#pragma unroll
                for (int e = 0; e < 8; ++e) x[8 * k + e] = (float)v[e];  // widening is exact
            }
            return;
        }
    }
#pragma unroll
    for (int k = 0; k < D; ++k) x[k] = (float)row[k];
}

// Eq. 2 for the range [lo, hi] on a row held in registers.  With TAIL the row has d elements,
// D - 8 < d < D: the last few registers hold no element and their terms are dropped.  (Padding the
// tree with zeros up to a larger power of two changes no sum, so D's tree serves d.)
template <int D, bool TAIL>
__device__ __forceinline__ float range_loss(const float (&x)[D], float lo, float hi, float qmax, int d)
{
    const StoredParams p = stored_params(lo, hi, qmax);
    return tree_sq_err<0, next_pow2(D), D, TAIL, D - 7, true>(x, p, d, x);  // uniform mask: no factors
}

// The whole path for the row this lane owns: load, min/max, Algorithm 1, encode, store.
// TAIL: the dimension d is not a multiple of 8 (D - 8 < d < D); registers at and beyond d copy element 0,
// which leaves min and max alone, and are masked out of the loss and the codes.  d is the same for
// every lane, so the masks are scalar conditions.
template <int D, typename Tin, bool TAIL = false>
__device__ __forceinline__ void greedy_rpl_row(const GreedyArgs& a, int64_t row, int d = D, uint8_t* stage = nullptr)
{
    const bool live = row < a.rows;
    const int64_t r = live ? row : a.rows - 1;  // tail lanes redo the last row and store nothing

    float x[D];
    if constexpr (TAIL) {
        // the first D - 8 elements always exist and load like a row of that dimension
        const Tin* src = static_cast<const Tin*>(a.table) + r * a.row_stride;
        if constexpr (D > 8) {
            float head[D - 8];
            load_row<D - 8>(src, a.vec_loads != 0, head);
#pragma unroll
            for (int k = 0; k < D - 8; ++k) x[k] = head[k];
        }
#pragma unroll
        for (int k = D - 8; k < D; ++k) x[k] = (float)src[k < d ? k : 0];
    } else {
        load_row<D>(static_cast<const Tin*>(a.table) + r * a.row_stride, a.vec_loads != 0, x);
    }

    // Algorithm 1, lines 1-2: the starting range is the row's range.
    float lo0 = x[0], hi0 = x[0];
#pragma unroll
    for (int k = 1; k < D; ++k) {
        lo0 = __builtin_fminf(lo0, x[k]);
        hi0 = __builtin_fmaxf(hi0, x[k]);
    }
    // A row may hold zeros of both signs; which of them a zero bound is depends on the order of the
    // comparisons.  Zero bounds are +0 by definition (the stored bias would differ in its sign bit).
    lo0 = canonical_zero(lo0);
    hi0 = canonical_zero(hi0);

    float best_lo = lo0, best_hi = hi0;
    if (a.n_iter > 0) {  // uniform branch: ratio == 0 needs no scoring at all
        const float stepsize = (hi0 - lo0) / a.n_bins;
        float cur_lo = lo0, cur_hi = hi0;
        float best = range_loss<D, TAIL>(x, lo0, hi0, a.qmax, d);
        for (int it = 0; it < a.n_iter; ++it) {
            const float next_lo = cur_lo + stepsize;
            const float next_hi = cur_hi - stepsize;
            const float loss_l = range_loss<D, TAIL>(x, next_lo, cur_hi, a.qmax, d);
            const float loss_r = range_loss<D, TAIL>(x, cur_lo, next_hi, a.qmax, d);
            const bool left = loss_l < loss_r;  // a tie moves the upper bound
            cur_lo = left ? next_lo : cur_lo;
            cur_hi = left ? cur_hi : next_hi;
            const float cand = left ? loss_l : loss_r;
            const bool better = cand < best;  // strictly smaller replaces
            best = better ? cand : best;
            best_lo = better ? cur_lo : best_lo;  // the pair is remembered together
            best_hi = better ? cur_hi : best_hi;
        }
    }

    // Encode with the best range (Eq. 1) and pack 8/nbits codes per byte, first element lowest.
    const float scale32 = (best_hi - best_lo) / a.qmax;
    const uint16_t scale_bits = f16_bits(scale32);
    const uint16_t bias_bits = f16_bits(best_lo);
    const StoredParams p = params_from_bits(scale_bits, bias_bits, a.qmax);
    if (live) {
        a.scale_f16[row] = scale_bits;
        a.bias_f16[row] = bias_bits;
    }
    auto encode = [&](auto nb) {
        constexpr int NB = decltype(nb)::value;
        const int nbytes = TAIL ? (d * NB + 7) / 8 : D * NB / 8;  // bytes per row; rows are dense
        if constexpr (TAIL) {
            // into the wave's staging area, which mirrors its 64 dense rows; the kernel copies it out
            encode_chunks<NB, D, 0, true>(x, p, d, stage + (int)threadIdx.x * nbytes, 0u, true);
        } else {
            const uint32_t cls = (nbytes % 16 == 0 && a.vec_stores == 2) ? 2u : ((nbytes % 4 == 0 && a.vec_stores >= 1) ? 1u : 0u);
            encode_chunks<NB, D, 0, false>(x, p, d, a.codes + row * nbytes, cls, live);
        }
    };
    if (a.nbits == 4) encode(Idx<4>{});  // uniform branches
    else if (a.nbits == 8) encode(Idx<8>{});
    else encode(Idx<2>{});
}

// First row of the calling wave, given the first row of its workgroup.  A wave whose first row is beyond the table
// (in the table's last workgroup) has nothing to do.
__device__ __forceinline__ int64_t rpl_wave_first_row(int64_t block_first_row)
{
    return block_first_row + (int64_t)(threadIdx.x & ~63u);
}

template <int D, typename Tin>
__global__ void __launch_bounds__(kRplBlock) greedy_rpl_kernel(GreedyArgs a)
{
    const int64_t row0 = (int64_t)blockIdx.x * blockDim.x;  // 64 or 256 rows per workgroup, the launcher's choice
    if (rpl_wave_first_row(row0) >= a.rows) return;  // no barrier in this kernel
    greedy_rpl_row<D, Tin>(a, row0 + threadIdx.x);
}

// The same for a dimension d that is not a multiple of 8, D = d rounded up.
// Rows of d * nbits / 8 bytes are not multiples of 4 bytes long, so a lane cannot store its row in
// words; the workgroup's 256 rows are contiguous in memory, though, and start at a multiple of 256 bytes.
// Each lane packs its row into LDS (an image of those 256 rows, D bytes each) and the workgroup copies the
// image out 16 bytes per lane at a time.
template <int D, typename Tin>
__global__ void __launch_bounds__(kRplBlock) greedy_rpl_tail_kernel(GreedyArgs a, int32_t d)
{
    __shared__ __attribute__((aligned(16))) uint8_t stage[kRplBlock * D];  // D bytes per row cover 8-bit codes
    const int64_t row0 = (int64_t)blockIdx.x * kRplBlock;
    if (rpl_wave_first_row(row0) < a.rows) greedy_rpl_row<D, Tin, true>(a, row0 + threadIdx.x, d, stage);  // wave-uniform
    __syncthreads();
    const int nbytes = (d * a.nbits + 7) / 8;
    const int64_t rows_here = a.rows - row0 < kRplBlock ? a.rows - row0 : kRplBlock;
    const int total = (int)rows_here * nbytes;
    uint8_t* dst = a.codes + row0 * nbytes;
    if (a.vec_stores == 2) {  // 16-byte aligned buffer: 256 * nbytes keeps every workgroup's start aligned
        for (int off = (int)threadIdx.x * 16; off < total; off += kRplBlock * 16) {
            if (off + 16 <= total) {
                *reinterpret_cast<uint4*>(dst + off) = *reinterpret_cast<const uint4*>(stage + off);
            } else {
                for (int b = off; b < total; ++b) dst[b] = stage[b];
            }
        }
    } else {
        for (int b = (int)threadIdx.x; b < total; b += kRplBlock) dst[b] = stage[b];
    }
}

// Several tables of one dimension and input type in one launch (a table takes ceil(rows / rows_per_block) workgroups):
// workgroup b belongs to the first table whose block_end exceeds b.  Small tables then share the chip with large ones instead of
// each waiting for a launch of its own to drain.
template <int D, typename Tin>
__global__ void __launch_bounds__(kRplBlock) greedy_rpl_group_kernel(GreedyGroup g)
{
    static_assert((kMaxGroupTables & (kMaxGroupTables - 1)) == 0 && sizeof(GreedyGroup) <= 4096, "see e4q_launch.h");
    // t = number of tables that end at or before this workgroup: a bisection over the running totals (entries beyond
    // the last table hold the grand total, which no workgroup number reaches).  Uniform: six scalar steps.
    int t = 0;
#pragma unroll
    for (int step = kMaxGroupTables / 2; step >= 1; step /= 2)
        if (blockIdx.x >= g.block_end[t + step - 1]) t += step;
    const uint32_t first_block = t == 0 ? 0u : g.block_end[t - 1];
    const GreedyTable& e = g.tables[t];
    GreedyArgs a;
    a.table = e.table;
    a.rows = e.rows;
    a.row_stride = e.row_stride;
    a.n_iter = g.n_iter;
    a.n_bins = g.n_bins;
    a.nbits = g.nbits;
    a.qmax = g.qmax;
    a.codes = e.codes;
    a.scale_f16 = e.scale_f16;
    a.bias_f16 = e.bias_f16;
    a.vec_loads = e.vec_loads;
    a.vec_stores = e.vec_stores;
    a.rpl_waves = 0u;  // host-side field
    const int64_t row0 = (int64_t)(blockIdx.x - first_block) * blockDim.x;
    if (rpl_wave_first_row(row0) >= a.rows) return;  // no barrier in this kernel
    greedy_rpl_row<D, Tin>(a, row0 + threadIdx.x);
}

template <int D, typename Tin>
inline hipError_t launch_greedy_rpl_group(const GreedyGroup& g, hipStream_t stream)
{
    const uint32_t blocks = g.block_end[g.n_tables - 1];
    if (g.rows_per_block != 64 && g.rows_per_block != kRplBlock) return hipErrorInvalidValue;
    hipLaunchKernelGGL((greedy_rpl_group_kernel<D, Tin>), dim3(blocks), dim3((unsigned)g.rows_per_block), 0, stream, g);
    return hipGetLastError();
}

// Host-side launcher for one (D, Tin) instantiation.  One work-item per row (rounded up to whole workgroups of 64 or
// 256), at most 2^31 + 255, which one grid dimension holds.
template <int D, typename Tin>
inline hipError_t launch_greedy_rpl(const GreedyArgs& a, hipStream_t stream)
{
    const int64_t block = rpl_rows_per_block(a.rows, a.rpl_waves);
    const int64_t blocks = (a.rows + block - 1) / block;
    hipLaunchKernelGGL((greedy_rpl_kernel<D, Tin>), dim3((unsigned)blocks), dim3((unsigned)block), 0, stream, a);
    return hipGetLastError();
}

// Needs D - 8 < d < D.
template <int D, typename Tin>
inline hipError_t launch_greedy_rpl_tail(const GreedyArgs& a, int32_t d, hipStream_t stream)
{
    if (d <= D - 8 || d >= D) return hipErrorInvalidValue;
    const int64_t blocks = (a.rows + kRplBlock - 1) / kRplBlock;
    hipLaunchKernelGGL((greedy_rpl_tail_kernel<D, Tin>), dim3((unsigned)blocks), dim3(kRplBlock), 0, stream, a, d);
    return hipGetLastError();
}

}  // namespace e4q
