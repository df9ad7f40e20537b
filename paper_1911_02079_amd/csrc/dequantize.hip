// De-quantization x_float = scale * x_int + bias (the sentence after Eq. 1).
//
// Bound by HBM: d/2 + 4 bytes in, 4d bytes out per row.
#include "e4q_device.h"
#include "e4q_index.h"
#include "e4q_launch.h"

namespace e4q {

constexpr int kDqBlock = 256;
typedef float floatx4 __attribute__((ext_vector_type(4)));

// dim % 4 == 0, codes aligned to the 4-element group (NBITS/2 bytes), out 16-byte aligned.  One
// thread per 4 elements: a wave reads contiguous code bytes and writes 1 KiB of contiguous output
// per store instruction (full cache lines, so nothing is written twice).
template <int NBITS, bool WIDE>
__global__ void __launch_bounds__(kDqBlock) dequantize_w4_kernel(const void* __restrict__ codes,
                                                                const uint16_t* __restrict__ scale_f16,
                                                                const uint16_t* __restrict__ bias_f16,
                                                                int64_t n_quads, uint32_t quads_per_row,
                                                                floatx4* __restrict__ out)
{
    // One group of four elements per thread and no loop: neighbouring workgroups write neighbouring
    // memory (measured 20 % faster than a capped grid with a grid-stride loop).  WIDE selects
    // 64-bit index arithmetic for tables with 2^32 or more groups.
    const int64_t w = linear_block() * kDqBlock + threadIdx.x;
    if (w >= n_quads) return;
    const int64_t row = group_of<WIDE>(w, quads_per_row);
    const float scale = f16_bits_to_float(scale_f16[row]);
    const float bias = f16_bits_to_float(bias_f16[row]);
    uint32_t c;  // the four codes of this thread, NBITS each, first element lowest
    if constexpr (NBITS == 8) c = __builtin_nontemporal_load(static_cast<const uint32_t*>(codes) + w);
    else if constexpr (NBITS == 4) c = __builtin_nontemporal_load(static_cast<const uint16_t*>(codes) + w);
    else c = __builtin_nontemporal_load(static_cast<const uint8_t*>(codes) + w);
    constexpr uint32_t kMask = (1u << NBITS) - 1u;
    floatx4 v;
    v.x = __builtin_fmaf((float)(c & kMask), scale, bias);
    v.y = __builtin_fmaf((float)((c >> NBITS) & kMask), scale, bias);
    v.z = __builtin_fmaf((float)((c >> (2 * NBITS)) & kMask), scale, bias);
    v.w = __builtin_fmaf((float)((c >> (3 * NBITS)) & kMask), scale, bias);
    __builtin_nontemporal_store(v, out + w);
}

// Any dim and alignment.  One thread per output element.
__global__ void __launch_bounds__(kDqBlock) dequantize_any_kernel(const uint8_t* __restrict__ codes,
                                                                 const uint16_t* __restrict__ scale_f16,
                                                                 const uint16_t* __restrict__ bias_f16,
                                                                 int64_t n_elems, uint32_t dim, uint32_t nbits,
                                                                 float* __restrict__ out)
{
    const uint32_t per = 8 / nbits;
    const uint32_t nbytes = (dim + per - 1) / per;
    const uint32_t mask = (1u << nbits) - 1u;
    const int64_t stride = (int64_t)gridDim.x * gridDim.y * kDqBlock;
    for (int64_t e = linear_block() * kDqBlock + threadIdx.x; e < n_elems; e += stride) {
        const int64_t row = e / dim;
        const uint32_t k = (uint32_t)(e - row * dim);
        const uint32_t byte = codes[row * nbytes + k / per];
        const uint32_t q = (byte >> ((k % per) * nbits)) & mask;
        out[e] = __builtin_fmaf((float)q, f16_bits_to_float(scale_f16[row]), f16_bits_to_float(bias_f16[row]));
    }
}

// Any dim >= 4, out 16-byte aligned: one thread per four consecutive elements of the flattened output (they
// may straddle one row boundary), one 16-byte store per lane.  The row and column of the first element
// cost one division (32-bit unless the table has 2^32 elements or more).  The four codes lie within 32
// bits of the code array, row padding included (at most 3 codes, 7 bits of padding and 7 bits of offset
// in the first byte ahead of the last code), so one unaligned 4-byte read fetches them; the threads
// whose read would pass the end of the array, or whose elements pass the end of the table, take the codes
// byte by byte.
template <bool WIDE>
__global__ void __launch_bounds__(kDqBlock) dequantize_flat4_kernel(const uint8_t* __restrict__ codes,
                                                                   const uint16_t* __restrict__ scale_f16,
                                                                   const uint16_t* __restrict__ bias_f16,
                                                                   int64_t n_elems, int64_t n_code_bytes, uint32_t dim,
                                                                   uint32_t nbits, float* __restrict__ out)
{
    const int64_t e0 = (linear_block() * kDqBlock + threadIdx.x) * 4;
    if (e0 >= n_elems) return;
    const uint32_t per = 8 / nbits;
    const uint32_t nbytes = (dim + per - 1) / per;
    const uint32_t mask = (1u << nbits) - 1u;
    const int64_t row = group_of<WIDE>(e0, dim);
    const uint32_t k = offset_in_group(e0, row, dim);
    const uint64_t bit0 = (uint64_t)k * nbits;  // of the first code within its row
    const int64_t byte0 = row * nbytes + (int64_t)(bit0 / 8);
    if (e0 + 4 <= n_elems && byte0 + 4 <= n_code_bytes) {
        uint32_t w;  // one unaligned 4-byte read (the aligned 8 bytes around it, shifted, measured 25 % slower)
        __builtin_memcpy(&w, codes + byte0, 4);
        w >>= (uint32_t)(bit0 % 8);
        const uint32_t in_row = dim - k;                    // elements of this row among the four, if < 4
        const uint32_t pad_bits = nbytes * 8 - dim * nbits;  // unused bits at the end of a row
        float scale = f16_bits_to_float(scale_f16[row]), bias = f16_bits_to_float(bias_f16[row]);
        float scale_next = scale, bias_next = bias;
        if (in_row < 4) {
            scale_next = f16_bits_to_float(scale_f16[row + 1]);
            bias_next = f16_bits_to_float(bias_f16[row + 1]);
        }
        float v[4];
#pragma unroll
        for (uint32_t j = 0; j < 4; ++j) {
            const bool next = j >= in_row;
            const uint32_t q = (w >> (j * nbits + (next ? pad_bits : 0u))) & mask;
            v[j] = __builtin_fmaf((float)q, next ? scale_next : scale, next ? bias_next : bias);
        }
        floatx4 o = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<floatx4*>(out + e0));
        return;
    }
    int64_t r = row;
    uint32_t c = k;
    for (int j = 0; j < 4 && e0 + j < n_elems; ++j) {
        const uint32_t byte = codes[r * nbytes + c / per];
        const uint32_t q = (byte >> ((c % per) * nbits)) & mask;
        out[e0 + j] = __builtin_fmaf((float)q, f16_bits_to_float(scale_f16[r]), f16_bits_to_float(bias_f16[r]));
        if (++c == dim) {
            c = 0;
            ++r;
        }
    }
}

template <int NBITS>
static void launch_w4(const void* codes, const uint16_t* scale_f16, const uint16_t* bias_f16, int64_t n_quads,
                      uint32_t quads_per_row, floatx4* out, hipStream_t stream)
{
    const dim3 grid = grid_for(blocks_for(n_quads, kDqBlock)), block(kDqBlock);
    if (needs_wide_index(n_quads))
        hipLaunchKernelGGL((dequantize_w4_kernel<NBITS, true>), grid, block, 0, stream, codes, scale_f16, bias_f16,
                           n_quads, quads_per_row, out);
    else
        hipLaunchKernelGGL((dequantize_w4_kernel<NBITS, false>), grid, block, 0, stream, codes, scale_f16, bias_f16,
                           n_quads, quads_per_row, out);
}

hipError_t launch_dequantize(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16,
                             int64_t rows, int32_t dim, int32_t nbits, float* out, hipStream_t stream)
{
    const uintptr_t group_bytes = nbits == 8 ? 4 : (nbits == 4 ? 2 : 1);
    const int64_t n_quads = rows * (dim / 4);
    const bool fast = dim % 4 == 0 && (reinterpret_cast<uintptr_t>(codes) % group_bytes == 0) &&
                      (reinterpret_cast<uintptr_t>(out) % 16 == 0) &&
                      blocks_for(n_quads, kDqBlock) >= 0;
    if (fast) {
        floatx4* o4 = reinterpret_cast<floatx4*>(out);
        const uint32_t qpr = (uint32_t)(dim / 4);
        if (nbits == 8) launch_w4<8>(codes, scale_f16, bias_f16, n_quads, qpr, o4, stream);
        else if (nbits == 4) launch_w4<4>(codes, scale_f16, bias_f16, n_quads, qpr, o4, stream);
        else launch_w4<2>(codes, scale_f16, bias_f16, n_quads, qpr, o4, stream);
    } else {
        const int64_t n_elems = rows * dim;
        const int64_t blocks4 = blocks_for((n_elems + 3) / 4, kDqBlock);
        if (reinterpret_cast<uintptr_t>(out) % 16 == 0 && blocks4 >= 0 && dim >= 4) {
            const int64_t n_code_bytes = rows * (((int64_t)dim * nbits + 7) / 8);
            if (needs_wide_index(n_elems))
                hipLaunchKernelGGL(dequantize_flat4_kernel<true>, grid_for(blocks4), dim3(kDqBlock), 0, stream,
                                   codes, scale_f16, bias_f16, n_elems, n_code_bytes, (uint32_t)dim, (uint32_t)nbits,
                                   out);
            else
                hipLaunchKernelGGL(dequantize_flat4_kernel<false>, grid_for(blocks4), dim3(kDqBlock), 0, stream,
                                   codes, scale_f16, bias_f16, n_elems, n_code_bytes, (uint32_t)dim, (uint32_t)nbits,
                                   out);
        } else {
            int64_t blocks = (n_elems + kDqBlock - 1) / kDqBlock;
            if (blocks > kMaxGridX) blocks = kMaxGridX;  // the kernel loops over what is left
            hipLaunchKernelGGL(dequantize_any_kernel, grid_for(blocks), dim3(kDqBlock), 0, stream, codes,
                               scale_f16, bias_f16, n_elems, (uint32_t)dim, (uint32_t)nbits, out);
        }
    }
    return hipGetLastError();
}

}  // namespace e4q
