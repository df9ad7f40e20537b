// Codebook kernels that are not specialised by dimension: the any-dimension Lloyd kernel, the
// dispatcher, and the codebook de-quantizer.
#include "kmeans16.h"

namespace e4q {

bool launch_kmeans16_rpl_f32(const KMeansArgs& a, int32_t dim, hipStream_t stream);
bool launch_kmeans16_rpl_f16(const KMeansArgs& a, int32_t dim, hipStream_t stream);
bool launch_kmeans16_rpl_tail_f32(const KMeansArgs& a, int32_t dim, hipStream_t stream);
bool launch_kmeans16_rpl_tail_f16(const KMeansArgs& a, int32_t dim, hipStream_t stream);

// Any dimension: one row per lane, elements re-read from memory in every round.
template <typename Tin>
__global__ void __launch_bounds__(64) kmeans16_any_kernel(KMeansArgs a, int32_t d)
{
    __shared__ LloydScratch scratch;
    const int lane = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * 64 + lane;
    if (row >= a.rows) return;  // no barriers in this kernel
    const Tin* src = static_cast<const Tin*>(a.table) + row * a.row_stride;
    uint16_t* cb = a.centroids_f16 + row * kK;
    const int nbytes = (d + 1) / 2;
    uint8_t* out = a.idx + row * nbytes;

    if (d <= kK) {  // every value is its own codebook entry
        for (int k = 0; k < kK; ++k) cb[k] = k < d ? f16_bits((float)src[k]) : (uint16_t)0;
        for (int b = 0; b < nbytes; ++b) out[b] = (uint8_t)((2 * b) | ((2 * b + 1 < d ? 2 * b + 1 : 0) << 4));
        return;
    }

    float lo = (float)src[0], hi = lo;
    for (int e = 1; e < d; ++e) {
        const float v = (float)src[e];
        lo = __builtin_fminf(lo, v);
        hi = __builtin_fmaxf(hi, v);
    }
    float c[kK];
    grid_centres(lo, hi, c);
    for (int it = 0; it < a.lloyd_iters; ++it) {
        lloyd_clear(scratch, lane);
        if (!a.force_scan && wave_centres_sorted(c)) {  // uniform over the wave's live lanes
            for (int e = 0; e < d; ++e) {
                const float v = (float)src[e];
                lloyd_add(scratch, lane, nearest_centre_sorted(v, c), v);
            }
        } else {
            for (int e = 0; e < d; ++e) {
                const float v = (float)src[e];
                lloyd_add(scratch, lane, nearest_centre(v, c), v);
            }
        }
        lloyd_update(scratch, lane, c);
    }
    float ch[kK];
#pragma unroll
    for (int k = 0; k < kK; ++k) {
        cb[k] = f16_bits(c[k]);
        ch[k] = through_f16(c[k]);
    }
    if (!a.force_scan && wave_centres_sorted(ch)) {
        for (int b = 0; b < nbytes; ++b) {
            const uint32_t q0 = (uint32_t)nearest_centre_sorted((float)src[2 * b], ch);
            const uint32_t q1 = (2 * b + 1 < d) ? (uint32_t)nearest_centre_sorted((float)src[2 * b + 1], ch) : 0u;
            out[b] = (uint8_t)(q0 | (q1 << 4));
        }
    } else {
        for (int b = 0; b < nbytes; ++b) {
            const uint32_t q0 = (uint32_t)nearest_centre((float)src[2 * b], ch);
            const uint32_t q1 = (2 * b + 1 < d) ? (uint32_t)nearest_centre((float)src[2 * b + 1], ch) : 0u;
            out[b] = (uint8_t)(q0 | (q1 << 4));
        }
    }
}

hipError_t launch_kmeans16(const KMeansArgs& a, int dtype, int32_t dim, hipStream_t stream)
{
    bool done = dtype == 0 ? launch_kmeans16_rpl_f32(a, dim, stream) : launch_kmeans16_rpl_f16(a, dim, stream);
    if (!done) done = dtype == 0 ? launch_kmeans16_rpl_tail_f32(a, dim, stream) : launch_kmeans16_rpl_tail_f16(a, dim, stream);
    if (!done) {
        const dim3 grid((unsigned)((a.rows + 63) / 64)), block(64);
        if (dtype == 0)
            hipLaunchKernelGGL(kmeans16_any_kernel<float>, grid, block, 0, stream, a, dim);
        else
            hipLaunchKernelGGL(kmeans16_any_kernel<_Float16>, grid, block, 0, stream, a, dim);
    }
    return hipGetLastError();
}

// Codebook dequantizer: out[r][k] = codebook[r][index[r][k]].  Bound by HBM (d/2 + 32 bytes in,
// 4d out per row); dim % 4 == 0 takes one 16-byte store per thread.
constexpr int kCbBlock = 256;
typedef float floatx4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(kCbBlock) dequantize_codebook_w4_kernel(const uint16_t* __restrict__ idx,
                                                                          const uint16_t* __restrict__ cb,
                                                                          int64_t n_quads, uint32_t quads_per_row,
                                                                          floatx4* __restrict__ out)
{
    // one group of four elements per thread, no loop (the host keeps n_quads below 2^32)
    const int64_t w = (int64_t)blockIdx.x * kCbBlock + threadIdx.x;
    if (w >= n_quads) return;
    const int64_t row = (int64_t)((uint32_t)w / quads_per_row);
    const uint16_t* book = cb + row * kK;
    const uint32_t q = __builtin_nontemporal_load(idx + w);
    floatx4 v;
    v.x = f16_bits_to_float(book[q & 15u]);
    v.y = f16_bits_to_float(book[(q >> 4) & 15u]);
    v.z = f16_bits_to_float(book[(q >> 8) & 15u]);
    v.w = f16_bits_to_float(book[q >> 12]);
    __builtin_nontemporal_store(v, out + w);
}

__global__ void __launch_bounds__(kCbBlock) dequantize_codebook_any_kernel(const uint8_t* __restrict__ idx,
                                                                           const uint16_t* __restrict__ cb,
                                                                           int64_t n_elems, uint32_t dim,
                                                                           float* __restrict__ out)
{
    const uint32_t nbytes = (dim + 1) / 2;
    const int64_t stride = (int64_t)gridDim.x * kCbBlock;
    for (int64_t e = (int64_t)blockIdx.x * kCbBlock + threadIdx.x; e < n_elems; e += stride) {
        const int64_t row = e / dim;
        const uint32_t k = (uint32_t)(e - row * dim);
        const uint32_t byte = idx[row * nbytes + k / 2];
        const uint32_t q = (k & 1u) ? (byte >> 4) : (byte & 15u);
        out[e] = f16_bits_to_float(cb[row * kK + q]);
    }
}

// Any dim, out 16-byte aligned: four consecutive elements of the flattened output per thread (they may
// straddle a row boundary), one 16-byte store per lane, one division per thread.
template <bool WIDE>
__global__ void __launch_bounds__(kCbBlock) dequantize_codebook_flat4_kernel(const uint8_t* __restrict__ idx,
                                                                             const uint16_t* __restrict__ cb,
                                                                             int64_t n_elems, uint32_t dim,
                                                                             float* __restrict__ out)
{
    const int64_t e0 = ((int64_t)blockIdx.x * kCbBlock + threadIdx.x) * 4;
    if (e0 >= n_elems) return;
    const uint32_t nbytes = (dim + 1) / 2;
    int64_t row = WIDE ? e0 / dim : (int64_t)((uint32_t)e0 / dim);
    uint32_t k = (uint32_t)(e0 - row * dim);
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        v[j] = 0.0f;
        if (e0 + j < n_elems) {
            const uint32_t byte = idx[row * nbytes + k / 2];
            const uint32_t q = (k & 1u) ? (byte >> 4) : (byte & 15u);
            v[j] = f16_bits_to_float(cb[row * kK + q]);
        }
        if (++k == dim) {
            k = 0;
            ++row;
        }
    }
    if (e0 + 4 <= n_elems) {
        floatx4 o = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<floatx4*>(out + e0));
    } else {
        for (int j = 0; e0 + j < n_elems; ++j) out[e0 + j] = v[j];
    }
}

hipError_t launch_dequantize_codebook(const uint8_t* idx, const uint16_t* centroids_f16, int64_t rows,
                                      int32_t dim, float* out, hipStream_t stream)
{
    const int64_t n_quads = rows * (dim / 4);
    const bool fast = dim % 4 == 0 && reinterpret_cast<uintptr_t>(idx) % 2 == 0 &&
                      reinterpret_cast<uintptr_t>(out) % 16 == 0 && n_quads <= 0xffffffffLL;
    if (fast) {
        const int64_t blocks = (n_quads + kCbBlock - 1) / kCbBlock;
        hipLaunchKernelGGL(dequantize_codebook_w4_kernel, dim3((unsigned)blocks), dim3(kCbBlock), 0, stream,
                           reinterpret_cast<const uint16_t*>(idx), centroids_f16, n_quads, (uint32_t)(dim / 4),
                           reinterpret_cast<floatx4*>(out));
    } else {
        const int64_t n_elems = rows * dim;
        const int64_t blocks4 = ((n_elems + 3) / 4 + kCbBlock - 1) / kCbBlock;
        if (reinterpret_cast<uintptr_t>(out) % 16 == 0 && blocks4 <= 0x7fffffffLL) {
            if (n_elems > 0xffffffffLL)
                hipLaunchKernelGGL(dequantize_codebook_flat4_kernel<true>, dim3((unsigned)blocks4), dim3(kCbBlock), 0,
                                   stream, idx, centroids_f16, n_elems, (uint32_t)dim, out);
            else
                hipLaunchKernelGGL(dequantize_codebook_flat4_kernel<false>, dim3((unsigned)blocks4), dim3(kCbBlock), 0,
                                   stream, idx, centroids_f16, n_elems, (uint32_t)dim, out);
        } else {
            int64_t blocks = (n_elems + kCbBlock - 1) / kCbBlock;
            if (blocks > 0x7fffffffLL) blocks = 0x7fffffffLL;  // the kernel loops over what is left
            hipLaunchKernelGGL(dequantize_codebook_any_kernel, dim3((unsigned)blocks), dim3(kCbBlock), 0, stream, idx,
                               centroids_f16, n_elems, (uint32_t)dim, out);
        }
    }
    return hipGetLastError();
}

}  // namespace e4q
