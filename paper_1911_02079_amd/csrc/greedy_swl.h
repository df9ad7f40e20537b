// Greedy clip search with L lanes per row ("sub-wave layout"): lane j of a row's group keeps the
// E contiguous elements [j*E, (j+1)*E) of the row in registers.
//
// The error sum of a range is an in-lane balanced tree over the lane's E elements followed by the upper
// levels of the same tree across the L lanes of the group (an xor-butterfly of DPP moves when L is a power of
// two, ds_bpermute steps for any other lane count); with contiguous chunks per lane that is exactly the
// balanced tree over index-adjacent pairs of the whole (zero padded) row, so results are bit
// identical to the one-row-per-lane kernels.  All L lanes of a group end up with the same sums and
// take the same decisions.
//
// Used where one row per lane is the wrong shape (the host weighs the layouts by a cost model):
//   * few rows (rows/64 waves would leave most of the chip idle): E = 8 spreads a row over up to
//     64 lanes;
//   * tables of a few waves per SIMD: E = 16, 32 or 64 gives every SIMD several waves to interleave,
//     which a lone wave per SIMD cannot make up for (it issues only every fifth cycle);
//   * ratio == 0 (plain min/max quantization, bound by HBM): with E = 8 a wave reads and writes
//     contiguous memory;
//   * dimensions above 224: E = 128 on ceil(dim / 128) lanes keeps the per-range scalar work (two short
//     divisions, two binary16 round trips, ~30 instructions that every lane of the group repeats) small
//     against 8 operations for each of 128 elements; E = 64 if the dimension is not a multiple of 8 (elements
//     that a lane may lack carry a mask factor in a register of their own).
// Masked instantiations take any dim <= E*L: elements at or beyond dim contribute exactly +0 to
// the sums and are kept out of min/max.  MASK = 0: dim == E*L, no masking; MASK = 1: dim is a
// multiple of 8, one select per block of 8 elements; MASK = 2: any dim, one mask factor per element;
// MASK = 3, 4, 5: the same for layouts in which every lane holds at least E/2, 3E/4, E - 8 elements (the
// fewest lanes that hold the row, whose last lane is at least that full): only the elements from there on
// carry a factor.
#pragma once

#include "e4q_device.h"
#include "e4q_index.h"
#include "e4q_launch.h"

namespace e4q {

constexpr int kSwlBlock = 256;

// Value of lane (id xor OFF).  DPP row operations inside 16 lanes, ds_bpermute beyond.
template <int OFF>
__device__ __forceinline__ float lane_xor(float v)
{
    const int i = __builtin_bit_cast(int, v);
    int r;
    if constexpr (OFF == 1) {
        r = __builtin_amdgcn_update_dpp(i, i, 0xB1, 0xF, 0xF, false);  // quad_perm [1,0,3,2]
    } else if constexpr (OFF == 2) {
        r = __builtin_amdgcn_update_dpp(i, i, 0x4E, 0xF, 0xF, false);  // quad_perm [2,3,0,1]
    } else if constexpr (OFF == 4) {
        // row_half_mirror (lane k <-> 7-k of each 8): the partner sits in the other quad, and after
        // the OFF = 1, 2 steps all lanes of a quad hold the same value
        r = __builtin_amdgcn_update_dpp(i, i, 0x141, 0xF, 0xF, false);
    } else if constexpr (OFF == 8) {
        r = __builtin_amdgcn_update_dpp(i, i, 0x140, 0xF, 0xF, false);  // row_mirror (k <-> 15-k)
    } else {
        r = __shfl_xor(i, OFF, 64);
    }
    return __builtin_bit_cast(float, r);
}

template <int L, class Op>
__device__ __forceinline__ float group_reduce(float v, Op op)
{
    if constexpr (L > 1) v = op(v, lane_xor<1>(v));
    if constexpr (L > 2) v = op(v, lane_xor<2>(v));
    if constexpr (L > 4) v = op(v, lane_xor<4>(v));
    if constexpr (L > 8) v = op(v, lane_xor<8>(v));
    if constexpr (L > 16) v = op(v, lane_xor<16>(v));
    if constexpr (L > 32) v = op(v, lane_xor<32>(v));
    return v;
}

// The same reductions for a group of `lanes` neighbouring lanes, any number from 2 to 64 (L = 0 in the
// templates below): lane `sub` of the group stands for leaf `sub` of a tree over next_pow2(lanes) leaves whose
// missing leaves are empty.  Step s adds node sub + s to node sub where sub is a multiple of 2s and the
// partner exists -- the adjacent pairs of the balanced tree, level by level -- and the group's first lane
// ends with the result, which every lane then reads.  Lane values travel by ds_bpermute.
__device__ __forceinline__ float lane_value(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane & 63) << 2, __builtin_bit_cast(int, v)));
}

// Sum of non-negative terms: a lane that takes nothing in a step adds +0.0f, which changes nothing.
__device__ __forceinline__ float group_sum_any(float v, int sub, int lanes)
{
    const int lane = (int)(threadIdx.x & 63u);
    for (int s = 1; s < lanes; s <<= 1) {
        const float t = lane_value(v, lane + s);
        const bool take = (sub & (2 * s - 1)) == 0 && sub + s < lanes;
        v = v + (take ? t : 0.0f);
    }
    return lane_value(v, lane - sub);
}

template <class Op>
__device__ __forceinline__ float group_reduce_any(float v, int sub, int lanes, Op op)
{
    const int lane = (int)(threadIdx.x & 63u);
    for (int s = 1; s < lanes; s <<= 1) {
        const float t = lane_value(v, lane + s);
        const bool take = (sub & (2 * s - 1)) == 0 && sub + s < lanes;
        v = take ? op(v, t) : v;
    }
    return lane_value(v, lane - sub);
}

// Elements of a lane below this index exist in every lane of the layout.
constexpr int swl_valid_below(int E, int MASK) { return MASK == 3 ? E / 2 : MASK == 4 ? 3 * E / 4 : MASK == 5 ? E - 8 : 0; }

template <int E, int L, int MASK>
__device__ __forceinline__ float swl_range_loss(const float (&x)[E], const float (&keep)[E], int nvalid, float lo,
                                                float hi, float qmax, int sub, int lanes)
{
    const StoredParams p = stored_params(lo, hi, qmax);
    float part;
    if constexpr (MASK == 1) {
        // tree over blocks of 8 of trees over 8 elements: the same balanced tree, masked per block
        const int nblocks = nvalid / 8;
        part = tree_sum<0, E / 8, E / 8>([&](auto b) {
            constexpr int blk = decltype(b)::value;
            const float bs = tree_sq_err<8 * blk, 8, E, false>(x, p, E, keep);
            return (blk < nblocks) ? bs : 0.0f;
        });
    } else {
        part = tree_sq_err<0, E, E, MASK >= 2, swl_valid_below(E, MASK)>(x, p, nvalid, keep);
    }
    if constexpr (L == 0) return group_sum_any(part, sub, lanes);
    else return group_reduce<L>(part, [](float a, float b) { return a + b; });
}

// L = 0: `lanes` lanes per row, a run-time number that need not be a power of two; a wave then holds
// 64 / lanes rows and its last 64 % lanes lanes idle (they redo a row and store nothing).
//
// TWIN (L a power of two up to 32): a row has two groups of L lanes, each holding the whole row, and the two
// ranges that Algorithm 1 scores per trip are scored at the same time, the left candidate by the first group and the
// right one by the second; the groups swap their sums and take the same decision.  The arithmetic per row is the
// same (plus one load and one first range), the chain of dependent trips is half as long: for tables too small
// to give every SIMD two waves, where the duration of the kernel is the duration of one wave.
template <int E, int L, typename Tin, int MASK, bool TWIN = false>
__global__ void __launch_bounds__(kSwlBlock) greedy_swl_kernel(GreedyArgs a, int32_t d, int32_t lanes_rt)
{
    constexpr bool MASKED = MASK != 0;
    static_assert(E % 8 == 0 && (E & (E - 1)) == 0 && (L & (L - 1)) == 0 && L <= 64, "bad layout");
    static_assert(!TWIN || (L >= 1 && L <= 32), "two groups of L lanes must fit a wave");
    const int lanes = L != 0 ? L : lanes_rt;
    int sub;
    int64_t row0, row;
    bool live;
    bool second = false;  // TWIN: this lane belongs to the group that scores the right candidate
    if constexpr (L != 0) {
        constexpr int kGroup = TWIN ? 2 * L : L;
        constexpr int kRowsPerBlock = kSwlBlock / kGroup;
        sub = threadIdx.x % L;
        row0 = linear_block() * kRowsPerBlock;
        row = row0 + threadIdx.x / kGroup;
        live = true;
        if constexpr (TWIN) second = ((threadIdx.x / L) & 1u) != 0;
    } else {
        const int rows_per_wave = 64 / lanes;
        const int lane = (int)(threadIdx.x & 63u), wave = (int)(threadIdx.x >> 6);
        const int group = lane / lanes;
        sub = lane - group * lanes;
        row0 = linear_block() * (int64_t)(rows_per_wave * (kSwlBlock / 64));
        row = row0 + wave * rows_per_wave + group;
        live = group < rows_per_wave;
    }
    if (row0 >= a.rows) return;  // padding of a folded grid (no barrier in this kernel)
    live = live && row < a.rows;
    const int64_t r = live ? row : a.rows - 1;  // tail groups redo the last row and store nothing
    const int base = sub * E;
    const int nvalid = MASKED ? min(max(d - base, 0), E) : E;

    const Tin* src = static_cast<const Tin*>(a.table) + r * a.row_stride;
    float x[E];
    if constexpr (!MASKED) {
        if (a.vec_loads) {
            constexpr int VEC = 16 / sizeof(Tin);
            typedef Tin vec_t __attribute__((ext_vector_type(VEC)));
            const vec_t* v = reinterpret_cast<const vec_t*>(src + base);
#pragma unroll
            for (int k = 0; k < E / VEC; ++k) {
                const vec_t t = v[k];
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[VEC * k + e] = (float)t[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < E; ++e) x[e] = (float)src[base + e];
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) x[e] = (float)src[(e < nvalid) ? base + e : 0];  // pad with element 0
    }

    float lo0 = x[0], hi0 = x[0];
#pragma unroll
    for (int e = 1; e < E; ++e) {
        lo0 = __builtin_fminf(lo0, x[e]);
        hi0 = __builtin_fmaxf(hi0, x[e]);
    }
    if constexpr (L == 0) {
        lo0 = group_reduce_any(lo0, sub, lanes, [](float p, float q) { return __builtin_fminf(p, q); });
        hi0 = group_reduce_any(hi0, sub, lanes, [](float p, float q) { return __builtin_fmaxf(p, q); });
    } else {
        lo0 = group_reduce<L>(lo0, [](float p, float q) { return __builtin_fminf(p, q); });
        hi0 = group_reduce<L>(hi0, [](float p, float q) { return __builtin_fmaxf(p, q); });
    }
    lo0 = canonical_zero(lo0);  // zero bounds are +0 whichever zeros the row holds
    hi0 = canonical_zero(hi0);

    // MASK >= 2: one factor per element that may be missing, 1.0f if it exists in this lane's part of the row
    // (see tree_sq_err)
    float keep[E];
    if constexpr (MASK >= 2) {
#pragma unroll
        for (int e = swl_valid_below(E, MASK); e < E; ++e) keep[e] = lane_keep_factor(e < nvalid);
    }

    float best_lo = lo0, best_hi = hi0;
    if (a.n_iter > 0) {
        const float stepsize = (hi0 - lo0) / a.n_bins;
        float cur_lo = lo0, cur_hi = hi0;
        float best = swl_range_loss<E, L, MASK>(x, keep, nvalid, lo0, hi0, a.qmax, sub, lanes);
        for (int it = 0; it < a.n_iter; ++it) {
            const float next_lo = cur_lo + stepsize;
            const float next_hi = cur_hi - stepsize;
            float loss_l, loss_r;
            if constexpr (TWIN) {
                const float mine = swl_range_loss<E, L, MASK>(x, keep, nvalid, second ? cur_lo : next_lo,
                                                              second ? next_hi : cur_hi, a.qmax, sub, lanes);
                const float theirs = lane_xor<L>(mine);  // the other group's lane at the same position
                loss_l = second ? theirs : mine;
                loss_r = second ? mine : theirs;
            } else {
                loss_l = swl_range_loss<E, L, MASK>(x, keep, nvalid, next_lo, cur_hi, a.qmax, sub, lanes);
                loss_r = swl_range_loss<E, L, MASK>(x, keep, nvalid, cur_lo, next_hi, a.qmax, sub, lanes);
            }
            const bool left = loss_l < loss_r;  // a tie moves the upper bound
            cur_lo = left ? next_lo : cur_lo;
            cur_hi = left ? cur_hi : next_hi;
            const float cand = left ? loss_l : loss_r;
            const bool better = cand < best;  // strictly smaller replaces
            best = better ? cand : best;
            best_lo = better ? cur_lo : best_lo;
            best_hi = better ? cur_hi : best_hi;
        }
    }

    const float scale32 = (best_hi - best_lo) / a.qmax;
    const uint16_t scale_bits = f16_bits(scale32);
    const uint16_t bias_bits = f16_bits(best_lo);
    const StoredParams p = params_from_bits(scale_bits, bias_bits, a.qmax);
    if constexpr (TWIN) live = live && !second;  // both groups hold the result; the first one stores it
    if (live && sub == 0) {
        a.scale_f16[row] = scale_bits;
        a.bias_f16[row] = bias_bits;
    }
    // Each lane packs and stores the codes of its own E elements (8/nbits per byte): E*nbits/8 bytes
    // at byte offset base*nbits/8 of the row, of which only the bytes that hold valid elements exist.
    auto encode = [&](auto nb) {
        constexpr int NB = decltype(nb)::value;
        constexpr int LANE_BYTES = E * NB / 8;
        const int row_bytes = (d * NB + 7) / 8;
        // word stores need 4-byte aligned pieces: a 4-byte aligned buffer, rows and lane pieces of 4k bytes
        const uint32_t cls = (a.vec_stores >= 1 && row_bytes % 4 == 0 && LANE_BYTES % 4 == 0) ? 1u : 0u;
        encode_chunks<NB, E, 0, MASKED>(x, p, nvalid, a.codes + row * row_bytes + base * NB / 8, cls, live);
    };
    if (a.nbits == 4) encode(Idx<4>{});  // uniform branches
    else if (a.nbits == 8) encode(Idx<8>{});
    else encode(Idx<2>{});
}

template <int E, int L, typename Tin, int MASK>
inline hipError_t launch_greedy_swl(const GreedyArgs& a, int32_t d, hipStream_t stream)
{
    constexpr int kRowsPerBlock = kSwlBlock / L;
    const int64_t blocks = (a.rows + kRowsPerBlock - 1) / kRowsPerBlock;
    hipLaunchKernelGGL((greedy_swl_kernel<E, L, Tin, MASK>), grid_for(blocks), dim3(kSwlBlock), 0, stream, a, d, L);
    return hipGetLastError();
}

// Two groups of L lanes per row (see TWIN above).
template <int E, int L, typename Tin, int MASK>
inline hipError_t launch_greedy_swl_twin(const GreedyArgs& a, int32_t d, hipStream_t stream)
{
    constexpr int kRowsPerBlock = kSwlBlock / (2 * L);
    const int64_t blocks = (a.rows + kRowsPerBlock - 1) / kRowsPerBlock;
    hipLaunchKernelGGL((greedy_swl_kernel<E, L, Tin, MASK, true>), grid_for(blocks), dim3(kSwlBlock), 0, stream, a, d, L);
    return hipGetLastError();
}

// `lanes` lanes per row, 2 .. 64, not necessarily a power of two.
template <int E, typename Tin, int MASK>
inline hipError_t launch_greedy_swl_any(const GreedyArgs& a, int32_t d, int32_t lanes, hipStream_t stream)
{
    if (lanes < 2 || lanes > 64 || (int64_t)E * lanes < d) return hipErrorInvalidValue;
    const int64_t rows_per_block = (64 / lanes) * (kSwlBlock / 64);
    const int64_t blocks = (a.rows + rows_per_block - 1) / rows_per_block;
    hipLaunchKernelGGL((greedy_swl_kernel<E, 0, Tin, MASK>), grid_for(blocks), dim3(kSwlBlock), 0, stream, a, d, lanes);
    return hipGetLastError();
}

// Dispatch over the (E, L) layouts that the including translation unit lists in E4Q_SWL_LAYOUTS.
// Its body differs between translation units, so it has internal linkage.  The mask mode follows
// from dim: none if dim == E*L, per block of 8 if dim % 8 == 0, else per element.
namespace {
template <typename Tin>
hipError_t dispatch_greedy_swl(const GreedyArgs& a, int32_t d, int E, int L, hipStream_t stream)
{
    const int mask = (d == E * L) ? 0 : (d % 8 == 0 ? 1 : 2);
    (void)mask;  // a translation unit may list no layout
#define E4Q_SWL(EE, LL)                                                              \
    if (E == EE && L == LL) {                                                        \
        if (mask == 0) return launch_greedy_swl<EE, LL, Tin, 0>(a, d, stream);       \
        if (mask == 1) return launch_greedy_swl<EE, LL, Tin, 1>(a, d, stream);       \
        return launch_greedy_swl<EE, LL, Tin, 2>(a, d, stream);                      \
    }
    E4Q_SWL_LAYOUTS
#undef E4Q_SWL
    return hipErrorInvalidValue;
}

// The same for the layouts with two groups per row that the translation unit lists in E4Q_SWL_TWIN_LAYOUTS.
#ifdef E4Q_SWL_TWIN_LAYOUTS
template <typename Tin>
hipError_t dispatch_greedy_swl_twin(const GreedyArgs& a, int32_t d, int E, int L, hipStream_t stream)
{
    const int mask = (d == E * L) ? 0 : (d % 8 == 0 ? 1 : 2);
#define E4Q_SWL_TWIN(EE, LL)                                                            \
    if (E == EE && L == LL) {                                                           \
        if (mask == 0) return launch_greedy_swl_twin<EE, LL, Tin, 0>(a, d, stream);     \
        if (mask == 1) return launch_greedy_swl_twin<EE, LL, Tin, 1>(a, d, stream);     \
        return launch_greedy_swl_twin<EE, LL, Tin, 2>(a, d, stream);                    \
    }
    E4Q_SWL_TWIN_LAYOUTS
#undef E4Q_SWL_TWIN
    return hipErrorInvalidValue;
}
#endif

// The same for a lane count that is not a power of two: E from the list in E4Q_SWL_ANY_E.
template <typename Tin>
hipError_t dispatch_greedy_swl_any(const GreedyArgs& a, int32_t d, int E, int lanes, hipStream_t stream)
{
    int mask = (d == E * lanes) ? 0 : (d % 8 == 0 ? 1 : 2);
    const int last = d - (lanes - 1) * E;  // elements in the row's last lane; every other lane is full if last > 0
    if (mask == 2 && E >= 32) mask = last >= E - 8 ? 5 : last >= 3 * E / 4 ? 4 : last >= E / 2 ? 3 : 2;
#define E4Q_SWL_E(EE)                                                                   \
    if (E == EE) {                                                                      \
        if (mask == 0) return launch_greedy_swl_any<EE, Tin, 0>(a, d, lanes, stream);   \
        if (mask == 1) return launch_greedy_swl_any<EE, Tin, 1>(a, d, lanes, stream);   \
        if constexpr (EE >= 32) {                                                       \
            if (mask == 3) return launch_greedy_swl_any<EE, Tin, 3>(a, d, lanes, stream); \
            if (mask == 4) return launch_greedy_swl_any<EE, Tin, 4>(a, d, lanes, stream); \
            if (mask == 5) return launch_greedy_swl_any<EE, Tin, 5>(a, d, lanes, stream); \
        }                                                                               \
        return launch_greedy_swl_any<EE, Tin, 2>(a, d, lanes, stream);                  \
    }
#ifdef E4Q_SWL_ANY_E
    E4Q_SWL_ANY_E
#endif
#undef E4Q_SWL_E
    return hipErrorInvalidValue;
}
}  // namespace

}  // namespace e4q
