// Greedy clip search for any embedding dimension: one table row per WAVE, row staged in LDS.
//
// This is the fallback for dimensions that have no register-resident instantiation.  A wave
// keeps the row (widened to binary32) in LDS, lane l scores elements l, l+64, ... of a
// candidate range, and the squared errors are reduced through LDS level by level over
// index-adjacent pairs, which is the same balanced tree the register-resident kernels build
// (zero padded to a power of two), so results are identical bit for bit.  All lanes of the wave
// compute the same scalar decisions redundantly; no atomics, one writer per output byte.
#include "e4q_device.h"
#include "e4q_launch.h"

namespace e4q {

constexpr int kWave = 64;

// Adjacent-pair tree over buf[0..p) (p a power of two), ping-ponging between two LDS buffers.
// Returns the total to every lane.  Workgroup = one wave; the barriers order LDS traffic.
__device__ __forceinline__ float lds_pair_tree(float* a, float* b, int p, int lane)
{
    float* src = a;
    float* dst = b;
    for (int m = p; m > 1; m >>= 1) {
        const int half = m >> 1;
        for (int i = lane; i < half; i += kWave) dst[i] = src[2 * i] + src[2 * i + 1];
        __syncthreads();
        float* t = src;
        src = dst;
        dst = t;
    }
    const float total = src[0];
    __syncthreads();  // everyone has read the total before the buffers are reused
    return total;
}

// Eq. 2 for [lo, hi] on the row in xs[0..d).
__device__ __forceinline__ float lds_range_loss(const float* xs, float* a, float* b, int d, int p,
                                                float lo, float hi, int lane)
{
    const StoredParams sp = stored_params(lo, hi);
    for (int k = lane; k < p; k += kWave) a[k] = (k < d) ? elem_sq_err(xs[k], sp) : 0.0f;
    __syncthreads();
    return lds_pair_tree(a, b, p, lane);
}

template <typename Tin>
__global__ void __launch_bounds__(kWave) greedy_generic_kernel(GreedyArgs g, int32_t d, int32_t p)
{
    extern __shared__ float lds[];
    float* xs = lds;       // p floats (d used)
    float* a = xs + p;     // p floats
    float* b = a + p;      // p/2 floats (at least 1)
    const int lane = threadIdx.x;
    const int nbytes = (d + 1) / 2;

    for (int64_t row = blockIdx.x; row < g.rows; row += gridDim.x) {
        const Tin* src = static_cast<const Tin*>(g.table) + row * g.row_stride;
        float lo0 = __builtin_inff(), hi0 = -__builtin_inff();
        for (int k = lane; k < d; k += kWave) {
            const float v = (float)src[k];
            xs[k] = v;
            lo0 = __builtin_fminf(lo0, v);
            hi0 = __builtin_fmaxf(hi0, v);
        }
        // wave-wide min/max (order does not matter for min/max)
        for (int off = kWave / 2; off > 0; off >>= 1) {
            lo0 = __builtin_fminf(lo0, __shfl_xor(lo0, off, kWave));
            hi0 = __builtin_fmaxf(hi0, __shfl_xor(hi0, off, kWave));
        }
        __syncthreads();

        float best_lo = lo0, best_hi = hi0;
        if (g.n_iter > 0) {
            const float stepsize = (hi0 - lo0) / g.n_bins;
            float cur_lo = lo0, cur_hi = hi0;
            float best = lds_range_loss(xs, a, b, d, p, lo0, hi0, lane);
            for (int it = 0; it < g.n_iter; ++it) {
                const float next_lo = cur_lo + stepsize;
                const float next_hi = cur_hi - stepsize;
                const float loss_l = lds_range_loss(xs, a, b, d, p, next_lo, cur_hi, lane);
                const float loss_r = lds_range_loss(xs, a, b, d, p, cur_lo, next_hi, lane);
                const bool left = loss_l < loss_r;
                cur_lo = left ? next_lo : cur_lo;
                cur_hi = left ? cur_hi : next_hi;
                const float cand = left ? loss_l : loss_r;
                const bool better = cand < best;
                best = better ? cand : best;
                best_lo = better ? cur_lo : best_lo;
                best_hi = better ? cur_hi : best_hi;
            }
        }

        const float scale32 = (best_hi - best_lo) / kQMax;
        const uint16_t scale_bits = f16_bits(scale32);
        const uint16_t bias_bits = f16_bits(best_lo);
        StoredParams sp;
        sp.scale = f16_bits_to_float(scale_bits);
        sp.bias = f16_bits_to_float(bias_bits);
        sp.inv = (sp.scale == 0.0f) ? 0.0f : 1.0f / sp.scale;
        uint8_t* out = g.codes + row * nbytes;
        for (int bidx = lane; bidx < nbytes; bidx += kWave) {
            const uint32_t q0 = (uint32_t)quantize_elem(xs[2 * bidx], sp);
            const uint32_t q1 = (2 * bidx + 1 < d) ? (uint32_t)quantize_elem(xs[2 * bidx + 1], sp) : 0u;
            out[bidx] = (uint8_t)(q0 | (q1 << 4));
        }
        if (lane == 0) {
            g.scale_f16[row] = scale_bits;
            g.bias_f16[row] = bias_bits;
        }
        __syncthreads();  // xs is overwritten by the next row
    }
}

hipError_t launch_greedy_generic(const GreedyArgs& g, int dtype, int32_t dim, hipStream_t stream)
{
    const int32_t p = next_pow2(dim);
    const size_t lds_bytes = sizeof(float) * ((size_t)2 * p + (p > 1 ? p / 2 : 1));
    int64_t blocks = g.rows;
    const int64_t cap = 256 * 32;  // resident waves on the chip; rows beyond are taken in a loop
    if (blocks > cap) blocks = cap;
    if (dtype == 0)
        hipLaunchKernelGGL(greedy_generic_kernel<float>, dim3((unsigned)blocks), dim3(kWave), lds_bytes, stream, g, dim, p);
    else
        hipLaunchKernelGGL(greedy_generic_kernel<_Float16>, dim3((unsigned)blocks), dim3(kWave), lds_bytes, stream, g, dim, p);
    return hipGetLastError();
}

}  // namespace e4q
