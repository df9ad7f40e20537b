// Host-visible launch interface between the C ABI (e4q_api.hip) and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace e4q {

// Arguments of every greedy-search kernel.  Pointers are device pointers.
struct GreedyArgs {
    const void* table;
    int64_t rows;
    int64_t row_stride;  // elements between rows
    int32_t n_iter;      // trips of Algorithm 1's loop (two candidate ranges per trip)
    float n_bins;        // b of Algorithm 1 as a float (divisor of the step size)
    uint8_t* codes;
    uint16_t* scale_f16;
    uint16_t* bias_f16;
    uint32_t vec_loads;   // 1: table base and row pitch are 16-byte aligned
    uint32_t vec_stores;  // 0: byte stores, 1: codes base 4-byte aligned, 2: 16-byte aligned
    int32_t nbits;        // 2, 4 or 8
    float qmax;           // 2^nbits - 1
    uint32_t rpl_waves;   // one-row-per-lane kernels: waves per workgroup, 1 or 4; 0: chosen from the row count
};

// Rows (= work-items) per workgroup of the one-row-per-lane kernels: 256 (four waves, one on each SIMD of a compute
// unit) while the launch has fewer than 8 waves per SIMD of the chip, 64 beyond (see greedy_rpl.h).  The kernels for
// dimensions that are not multiples of 8 stage their codes in LDS per workgroup and always take 256.
constexpr int kRplMaxRowsPerBlock = 256;
inline int rpl_rows_per_block(int64_t rows_in_launch) { return rows_in_launch >= (int64_t)8 * 1024 * 64 ? 64 : kRplMaxRowsPerBlock; }
// The same with the diagnostic override (waves per workgroup, 0 = none).
inline int rpl_rows_per_block(int64_t rows_in_launch, uint32_t forced_waves)
{
    return forced_waves == 1 ? 64 : forced_waves == 4 ? kRplMaxRowsPerBlock : rpl_rows_per_block(rows_in_launch);
}

// One launch over several tables of the same dimension and input type (one row per lane).
constexpr int kMaxGroupTables = 64;  // a power of two (the kernel bisects block_end); the group travels as a kernel argument, under 4 KiB
struct GreedyTable {
    const void* table;
    int64_t rows;
    int64_t row_stride;
    uint8_t* codes;
    uint16_t* scale_f16;
    uint16_t* bias_f16;
    uint32_t vec_loads;
    uint32_t vec_stores;
};
struct GreedyGroup {
    int32_t rows_per_block;  // 64 or 256 (rpl_rows_per_block of the launch's rows): the workgroup size
    int32_t n_tables;  // 1 .. kMaxGroupTables
    int32_t n_iter;
    float n_bins;
    int32_t nbits;
    float qmax;
    uint32_t block_end[kMaxGroupTables];  // running total of ceil(rows / rows_per_block) workgroups
    GreedyTable tables[kMaxGroupTables];
};

// Register-resident kernels exist for these dimensions: multiples of 8 up to 224 (the row and some thirty
// registers of working state must leave room for two waves per SIMD: 256 registers each).
inline bool rpl_supports_dim(int32_t dim) { return dim >= 8 && dim <= 224 && dim % 8 == 0; }
// The grouped (batch) launches are instantiated up to 128.
inline bool rpl_group_supports_dim(int32_t dim) { return dim >= 8 && dim <= 128 && dim % 8 == 0; }
// Row per lane with a masked tail: any other dimension below 224 (registers for the next multiple of 8).
inline bool rpl_tail_supports_dim(int32_t dim) { return dim >= 1 && dim < 224 && dim % 8 != 0; }

// Each returns hipGetLastError() after enqueueing.
hipError_t launch_greedy_rpl_f32(const GreedyArgs& a, int32_t dim, hipStream_t stream);
hipError_t launch_greedy_rpl_f16(const GreedyArgs& a, int32_t dim, hipStream_t stream);
hipError_t launch_greedy_rpl_wide_f32(const GreedyArgs& a, int32_t dim, hipStream_t stream);  // 136 .. 224
hipError_t launch_greedy_rpl_wide_f16(const GreedyArgs& a, int32_t dim, hipStream_t stream);
hipError_t launch_greedy_rpl_wide_tail_f32(const GreedyArgs& a, int32_t dim, hipStream_t stream);  // 129 .. 223, not 8k
hipError_t launch_greedy_rpl_wide_tail_f16(const GreedyArgs& a, int32_t dim, hipStream_t stream);
hipError_t launch_greedy_rpl_tail_f32(const GreedyArgs& a, int32_t dim, hipStream_t stream);
hipError_t launch_greedy_rpl_tail_f16(const GreedyArgs& a, int32_t dim, hipStream_t stream);
hipError_t launch_greedy_rpl_group_f32(const GreedyGroup& g, int32_t dim, hipStream_t stream);
hipError_t launch_greedy_rpl_group_f16(const GreedyGroup& g, int32_t dim, hipStream_t stream);
// Sub-wave layouts: L lanes per row, E contiguous elements per lane (see greedy_swl.h).
// "small": E in {8, 16}; "mid": E in {32, 64}; "big": E = 128.  L is a power of two up to 64 (32 for E = 128);
// needs dim <= E * L.
hipError_t launch_greedy_swl_f32_small(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream);
hipError_t launch_greedy_swl_f32_mid(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream);
hipError_t launch_greedy_swl_f32_big(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream);
hipError_t launch_greedy_swl_f16_small(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream);
hipError_t launch_greedy_swl_f16_mid(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream);
hipError_t launch_greedy_swl_f16_big(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream);
// Two groups of L lanes per row, one per candidate range of a trip: E in {8, 16}, L a power of two up to 32.
hipError_t launch_greedy_swl_twin_f32(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream);
hipError_t launch_greedy_swl_twin_f16(const GreedyArgs& a, int32_t dim, int E, int L, hipStream_t stream);
// The same with any number of lanes per row from 2 to 64 (a wave holds 64 / lanes rows): E in {8 .. 128}.
hipError_t launch_greedy_swl_any_f32(const GreedyArgs& a, int32_t dim, int E, int lanes, hipStream_t stream);
hipError_t launch_greedy_swl_any_f16(const GreedyArgs& a, int32_t dim, int E, int lanes, hipStream_t stream);

// Arguments of the codebook (16-means) kernels.
struct KMeansArgs {
    const void* table;
    int64_t rows;
    int64_t row_stride;  // elements between rows
    int32_t lloyd_iters;
    uint8_t* idx;
    uint16_t* centroids_f16;
    uint32_t vec_loads;   // 1: table base and row pitch are 16-byte aligned
    uint32_t vec_stores;  // >= 1: idx base is 4-byte aligned; 2: 16-byte aligned
    uint32_t force_scan;  // 1: always scan all 16 centres (diagnostic; results are identical)
    uint32_t waves;       // register-resident kernels: waves per workgroup, 1 or 4; 0: chosen from the row count
};
hipError_t launch_kmeans16(const KMeansArgs& a, int dtype, int32_t dim, hipStream_t stream);
hipError_t launch_dequantize_codebook(const uint8_t* idx, const uint16_t* centroids_f16, int64_t rows,
                                      int32_t dim, float* out, hipStream_t stream);
hipError_t launch_sparse_lengths_sum(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16,
                                     int64_t rows, int32_t dim, const void* indices, int32_t index_bytes,
                                     int64_t n_indices, const int64_t* offsets, int64_t n_bags, float* out,
                                     hipStream_t stream);
hipError_t launch_fuse_rows(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16, int64_t rows,
                            int32_t dim, int64_t row_pitch, uint8_t* fused, hipStream_t stream);
hipError_t launch_sparse_lengths_sum_fused(const uint8_t* fused, int64_t rows, int32_t dim, int64_t row_pitch,
                                           const void* indices, int32_t index_bytes, int64_t n_indices,
                                           const int64_t* offsets, int64_t n_bags, float* out, bool nontemporal,
                                           hipStream_t stream);
hipError_t launch_dequantize(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16,
                             int64_t rows, int32_t dim, int32_t nbits, float* out, hipStream_t stream);

}  // namespace e4q
