// Index arithmetic of the kernels that give one thread to a fixed-size group of outputs (four
// elements of a row, one code word of a bag): which row or bag a thread number belongs to.
// Tables of the paper's size (50 M rows of 128 values, Section 5) have more than 2^32 elements, so
// thread numbers are 64-bit; a 64-bit division costs several times a 32-bit one, so it is used only
// when a thread number can exceed 32 bits.  The functions are host-callable as well, so that a CPU
// test can check them at the 2^32 boundary.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace e4q {

// True when thread numbers 0 .. n_items - 1 do not all fit in 32 bits.
__host__ __device__ __forceinline__ bool needs_wide_index(int64_t n_items) { return n_items > 0x100000000LL; }

// t / per for 0 <= t < n_items, n_items as classified by needs_wide_index (WIDE = its result).
template <bool WIDE>
__host__ __device__ __forceinline__ int64_t group_of(int64_t t, uint32_t per)
{
    return WIDE ? t / (int64_t)per : (int64_t)((uint32_t)t / per);
}

// The same with the classification taken at run time (uniform across a launch).
__host__ __device__ __forceinline__ int64_t group_of(int64_t t, int64_t n_items, uint32_t per)
{
    return needs_wide_index(n_items) ? group_of<true>(t, per) : group_of<false>(t, per);
}

// Position of t inside its group.
__host__ __device__ __forceinline__ uint32_t offset_in_group(int64_t t, int64_t group, uint32_t per)
{
    return (uint32_t)(t - group * (int64_t)per);
}

// Launch shape.  The dispatch packet counts the WORK-ITEMS of each grid dimension in 32 bits, so
// workgroups * threads per workgroup must stay below 2^32 in every dimension; a larger
// one-dimensional launch is not refused, it silently runs a truncated grid.  Launches therefore put
// at most kMaxGridX workgroups in x (2^31 work-items even with 1024-thread workgroups) and fold the rest
// into y; kernels number their workgroups with linear_block() and return for numbers at or beyond
// the count they were launched for (the last row of a folded grid is padded).
constexpr int64_t kMaxGridX = 1 << 21;
constexpr int64_t kMaxGridY = 65535;

// Number of workgroups of `block` threads that cover n_items threads, or -1 if no launch can hold them.
__host__ __device__ __forceinline__ int64_t blocks_for(int64_t n_items, int32_t block)
{
    const int64_t b = (n_items + block - 1) / block;
    return b <= kMaxGridX * kMaxGridY ? b : -1;
}

// Grid for n_blocks workgroups, 1 <= n_blocks <= kMaxGridX * kMaxGridY.
inline dim3 grid_for(int64_t n_blocks)
{
    if (n_blocks <= kMaxGridX) return dim3((unsigned)n_blocks);
    return dim3((unsigned)kMaxGridX, (unsigned)((n_blocks + kMaxGridX - 1) / kMaxGridX));
}

// Number of this workgroup in a grid made by grid_for.
__device__ __forceinline__ int64_t linear_block() { return (int64_t)blockIdx.y * gridDim.x + blockIdx.x; }

}  // namespace e4q
