// Codebook kernels that are not specialised by dimension: the any-dimension Lloyd kernel, the
// dispatcher, and the codebook de-quantizer.
#include "kmeans16.h"
#include "e4q_index.h"

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
                lloyd_add_at(scratch, nearest_centre_sorted<512>(v, c) | (lane * 8), v);
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

// Dimensions above 128: one row per lane, 64 elements of it in registers at a time.  Every round walks
// the row chunk by chunk (16-byte loads where the table allows them), so a cluster's sum still grows
// in element order; the per-element work is the register-resident kernels' (bisection over ordered
// centres, scan otherwise).  A row is read 2 + lloyd_iters times instead of once; those reads mostly
// hit the caches and the path stays bound by VALU issue.
constexpr int kChunk = 64;

template <typename Tin>
__device__ __forceinline__ void load_chunk(const Tin* __restrict__ src, int n, bool vec, float (&x)[kChunk])
{
    if (n == kChunk) {
        load_row<kChunk>(src, vec, x);
    } else {
#pragma unroll
        for (int k = 0; k < kChunk; ++k) x[k] = (float)src[k < n ? k : 0];
    }
}

template <typename Tin>
__global__ void __launch_bounds__(64) kmeans16_chunk_kernel(KMeansArgs a, int32_t d)
{
    __shared__ LloydScratch scratch;
    const int lane = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * 64 + lane;
    const bool live = row < a.rows;
    const int64_t r = live ? row : a.rows - 1;  // tail lanes redo the last row and store nothing
    const Tin* src = static_cast<const Tin*>(a.table) + r * a.row_stride;
    // chunk starts are multiples of 64 elements, so they keep the row's 16-byte alignment
    const bool vec = a.vec_loads != 0;
    float x[kChunk];

    float lo = (float)src[0], hi = lo;
    for (int c0 = 0; c0 < d; c0 += kChunk) {
        const int n = d - c0 < kChunk ? d - c0 : kChunk;
        load_chunk(src + c0, n, vec, x);  // registers beyond n copy the chunk's first element
#pragma unroll
        for (int k = 0; k < kChunk; ++k) {
            lo = __builtin_fminf(lo, x[k]);
            hi = __builtin_fmaxf(hi, x[k]);
        }
    }
    float c[kK];
    grid_centres(lo, hi, c);

    for (int it = 0; it < a.lloyd_iters; ++it) {
        lloyd_clear(scratch, lane);
        if (!a.force_scan && wave_centres_sorted(c)) {
            for (int c0 = 0; c0 < d; c0 += kChunk) {
                const int n = d - c0 < kChunk ? d - c0 : kChunk;
                load_chunk(src + c0, n, vec, x);
                if (n == kChunk) {  // whole chunk: no test per element, so the elements' chains interleave
#pragma unroll
                    for (int e = 0; e < kChunk; ++e) lloyd_add_at(scratch, nearest_centre_sorted<512>(x[e], c) | (lane * 8), x[e]);
                } else {
#pragma unroll
                    for (int e = 0; e < kChunk; ++e)
                        if (e < n) lloyd_add_at(scratch, nearest_centre_sorted<512>(x[e], c) | (lane * 8), x[e]);  // scalar branch
                }
            }
        } else {
#pragma unroll 1
            for (int e = 0; e < d; ++e) {
                const float v = (float)src[e];
                lloyd_add(scratch, lane, nearest_centre(v, c), v);
            }
        }
        lloyd_update(scratch, lane, c);
    }

    float ch[kK];
#pragma unroll
    for (int k = 0; k < kK; ++k) ch[k] = through_f16(c[k]);
    if (live) store_codebook(c, a.centroids_f16 + row * kK);
    const int nbytes = (d + 1) / 2;
    uint8_t* out = a.idx + row * nbytes;
    if (a.force_scan || !wave_centres_sorted(ch)) {
        if (live) {
#pragma unroll 1
            for (int b = 0; b < nbytes; ++b) {
                const uint32_t q0 = (uint32_t)nearest_centre((float)src[2 * b], ch);
                const uint32_t q1 = (2 * b + 1 < d) ? (uint32_t)nearest_centre((float)src[2 * b + 1], ch) : 0u;
                out[b] = (uint8_t)(q0 | (q1 << 4));
            }
        }
        return;
    }
    // word stores need 4-byte aligned rows: a 4-byte aligned buffer and a row size of 4k bytes
    const bool words = a.vec_stores >= 1 && nbytes % 4 == 0;
    for (int c0 = 0; c0 < d; c0 += kChunk) {
        const int n = d - c0 < kChunk ? d - c0 : kChunk;
        load_chunk(src + c0, n, vec, x);
        uint32_t w[kChunk / 8];
#pragma unroll
        for (int i = 0; i < kChunk / 8; ++i) {
            uint32_t acc = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t q = (uint32_t)nearest_centre_sorted(x[8 * i + e], ch);
                acc |= (8 * i + e < n ? q : 0u) << (4 * e);
            }
            w[i] = acc;
        }
        if (!live) continue;
        const int chunk_bytes = (n + 1) / 2;
        uint8_t* o = out + c0 / 2;
        if (words && chunk_bytes % 4 == 0) {
#pragma unroll
            for (int i = 0; i < kChunk / 8; ++i)
                if (4 * i < chunk_bytes) reinterpret_cast<uint32_t*>(o)[i] = w[i];
        } else {
#pragma unroll
            for (int b = 0; b < kChunk / 2; ++b)
                if (b < chunk_bytes) o[b] = (uint8_t)(w[b / 4] >> (8 * (b % 4)));
        }
    }
}

hipError_t launch_kmeans16(const KMeansArgs& a, int dtype, int32_t dim, hipStream_t stream)
{
    bool done = dtype == 0 ? launch_kmeans16_rpl_f32(a, dim, stream) : launch_kmeans16_rpl_f16(a, dim, stream);
    if (!done) done = dtype == 0 ? launch_kmeans16_rpl_tail_f32(a, dim, stream) : launch_kmeans16_rpl_tail_f16(a, dim, stream);
    if (!done) {
        const dim3 grid((unsigned)((a.rows + 63) / 64)), block(64);
        if (dim > 128) {
            if (dtype == 0)
                hipLaunchKernelGGL(kmeans16_chunk_kernel<float>, grid, block, 0, stream, a, dim);
            else
                hipLaunchKernelGGL(kmeans16_chunk_kernel<_Float16>, grid, block, 0, stream, a, dim);
        } else {  // dim <= 16: a conversion
            if (dtype == 0)
                hipLaunchKernelGGL(kmeans16_any_kernel<float>, grid, block, 0, stream, a, dim);
            else
                hipLaunchKernelGGL(kmeans16_any_kernel<_Float16>, grid, block, 0, stream, a, dim);
        }
    }
    return hipGetLastError();
}

// Codebook dequantizer: out[r][k] = codebook[r][index[r][k]].  Bound by HBM (d/2 + 32 bytes in,
// 4d out per row); dim % 4 == 0 takes one 16-byte store per thread.
constexpr int kCbBlock = 256;
typedef float floatx4 __attribute__((ext_vector_type(4)));

template <bool WIDE>
__global__ void __launch_bounds__(kCbBlock) dequantize_codebook_w4_kernel(const uint16_t* __restrict__ idx,
                                                                          const uint16_t* __restrict__ cb,
                                                                          int64_t n_quads, uint32_t quads_per_row,
                                                                          floatx4* __restrict__ out)
{
    // one group of four elements per thread, no loop
    const int64_t w = linear_block() * kCbBlock + threadIdx.x;
    if (w >= n_quads) return;
    const int64_t row = group_of<WIDE>(w, quads_per_row);
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
    const int64_t stride = (int64_t)gridDim.x * gridDim.y * kCbBlock;
    for (int64_t e = linear_block() * kCbBlock + threadIdx.x; e < n_elems; e += stride) {
        const int64_t row = e / dim;
        const uint32_t k = (uint32_t)(e - row * dim);
        const uint32_t byte = idx[row * nbytes + k / 2];
        const uint32_t q = (k & 1u) ? (byte >> 4) : (byte & 15u);
        out[e] = f16_bits_to_float(cb[row * kK + q]);
    }
}

// Any dim >= 4, out 16-byte aligned: four consecutive elements of the flattened output per thread (they may
// straddle one row boundary), one 16-byte store per lane, one division per thread.  The four indices lie
// within 24 bits of the index array (a row of odd dimension ends in 4 unused bits), so one unaligned 4-byte
// read fetches them; threads whose read would pass the end of the array, or whose elements pass the end of
// the table, take them byte by byte.
template <bool WIDE>
__global__ void __launch_bounds__(kCbBlock) dequantize_codebook_flat4_kernel(const uint8_t* __restrict__ idx,
                                                                             const uint16_t* __restrict__ cb,
                                                                             int64_t n_elems, int64_t n_idx_bytes,
                                                                             uint32_t dim, float* __restrict__ out)
{
    const int64_t e0 = (linear_block() * kCbBlock + threadIdx.x) * 4;
    if (e0 >= n_elems) return;
    const uint32_t nbytes = (dim + 1) / 2;
    const int64_t row = group_of<WIDE>(e0, dim);
    const uint32_t k = offset_in_group(e0, row, dim);
    const int64_t byte0 = row * nbytes + k / 2;
    if (e0 + 4 <= n_elems && byte0 + 4 <= n_idx_bytes) {
        uint32_t w;
        __builtin_memcpy(&w, idx + byte0, 4);
        w >>= (k & 1u) * 4u;
        const uint32_t in_row = dim - k;               // elements of this row among the four, if < 4
        const uint32_t pad_bits = (dim & 1u) * 4u;     // unused bits at the end of a row
        const uint16_t* book = cb + row * kK;
        float v[4];
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
            const bool next = j >= in_row;
            const uint32_t q = (w >> (4u * j + (next ? pad_bits : 0u))) & 15u;
            v[j] = f16_bits_to_float(book[(next ? kK : 0) + q]);  // the next row's codebook follows this one's
        }
        floatx4 o = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<floatx4*>(out + e0));
        return;
    }
    int64_t r = row;
    uint32_t c = k;
    for (int j = 0; j < 4 && e0 + j < n_elems; ++j) {
        const uint32_t byte = idx[r * nbytes + c / 2];
        const uint32_t q = (c & 1u) ? (byte >> 4) : (byte & 15u);
        out[e0 + j] = f16_bits_to_float(cb[r * kK + q]);
        if (++c == dim) {
            c = 0;
            ++r;
        }
    }
}

hipError_t launch_dequantize_codebook(const uint8_t* idx, const uint16_t* centroids_f16, int64_t rows,
                                      int32_t dim, float* out, hipStream_t stream)
{
    const int64_t n_quads = rows * (dim / 4);
    const bool fast = dim % 4 == 0 && reinterpret_cast<uintptr_t>(idx) % 2 == 0 &&
                      reinterpret_cast<uintptr_t>(out) % 16 == 0 && blocks_for(n_quads, kCbBlock) >= 0;
    if (fast) {
        const dim3 grid = grid_for(blocks_for(n_quads, kCbBlock)), block(kCbBlock);
        if (needs_wide_index(n_quads))
            hipLaunchKernelGGL(dequantize_codebook_w4_kernel<true>, grid, block, 0, stream,
                               reinterpret_cast<const uint16_t*>(idx), centroids_f16, n_quads, (uint32_t)(dim / 4),
                               reinterpret_cast<floatx4*>(out));
        else
            hipLaunchKernelGGL(dequantize_codebook_w4_kernel<false>, grid, block, 0, stream,
                               reinterpret_cast<const uint16_t*>(idx), centroids_f16, n_quads, (uint32_t)(dim / 4),
                               reinterpret_cast<floatx4*>(out));
    } else {
        const int64_t n_elems = rows * dim;
        const int64_t blocks4 = blocks_for((n_elems + 3) / 4, kCbBlock);
        if (reinterpret_cast<uintptr_t>(out) % 16 == 0 && blocks4 >= 0 && dim >= 4) {
            const int64_t n_idx_bytes = rows * ((dim + 1) / 2);
            if (needs_wide_index(n_elems))
                hipLaunchKernelGGL(dequantize_codebook_flat4_kernel<true>, grid_for(blocks4), dim3(kCbBlock), 0,
                                   stream, idx, centroids_f16, n_elems, n_idx_bytes, (uint32_t)dim, out);
            else
                hipLaunchKernelGGL(dequantize_codebook_flat4_kernel<false>, grid_for(blocks4), dim3(kCbBlock), 0,
                                   stream, idx, centroids_f16, n_elems, n_idx_bytes, (uint32_t)dim, out);
        } else {
            int64_t blocks = (n_elems + kCbBlock - 1) / kCbBlock;
            if (blocks > kMaxGridX) blocks = kMaxGridX;  // the kernel loops over what is left
            hipLaunchKernelGGL(dequantize_codebook_any_kernel, grid_for(blocks), dim3(kCbBlock), 0, stream, idx,
                               centroids_f16, n_elems, (uint32_t)dim, out);
        }
    }
    return hipGetLastError();
}

}  // namespace e4q
