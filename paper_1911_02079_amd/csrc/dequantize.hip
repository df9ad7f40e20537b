// De-quantization x_float = scale * x_int + bias (the sentence after Eq. 1).
//
// Bound by HBM: d/2 + 4 bytes in, 4d bytes out per row.
#include "e4q_device.h"
#include "e4q_launch.h"

namespace e4q {

constexpr int kDqBlock = 256;
typedef float floatx4 __attribute__((ext_vector_type(4)));

// dim % 4 == 0, codes 2-byte aligned, out 16-byte aligned.  One thread per 4 elements: a wave
// reads 128 contiguous bytes of codes and writes 1 KiB of contiguous output per store instruction
// (full cache lines, so nothing is written twice).
__global__ void __launch_bounds__(kDqBlock) dequantize_w4_kernel(const uint16_t* __restrict__ codes,
                                                                const uint16_t* __restrict__ scale_f16,
                                                                const uint16_t* __restrict__ bias_f16,
                                                                int64_t n_quads, uint32_t quads_per_row,
                                                                floatx4* __restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * kDqBlock;
    for (int64_t w = (int64_t)blockIdx.x * kDqBlock + threadIdx.x; w < n_quads; w += stride) {
        const int64_t row = (n_quads <= 0xffffffffLL) ? (int64_t)((uint32_t)w / quads_per_row) : w / quads_per_row;
        const float scale = f16_bits_to_float(scale_f16[row]);
        const float bias = f16_bits_to_float(bias_f16[row]);
        const uint32_t c = __builtin_nontemporal_load(codes + w);
        floatx4 v;
        v.x = __builtin_fmaf((float)(c & 15u), scale, bias);
        v.y = __builtin_fmaf((float)((c >> 4) & 15u), scale, bias);
        v.z = __builtin_fmaf((float)((c >> 8) & 15u), scale, bias);
        v.w = __builtin_fmaf((float)(c >> 12), scale, bias);
        __builtin_nontemporal_store(v, out + w);
    }
}

// Any dim and alignment.  One thread per output element.
__global__ void __launch_bounds__(kDqBlock) dequantize_any_kernel(const uint8_t* __restrict__ codes,
                                                                 const uint16_t* __restrict__ scale_f16,
                                                                 const uint16_t* __restrict__ bias_f16,
                                                                 int64_t n_elems, uint32_t dim,
                                                                 float* __restrict__ out)
{
    const uint32_t nbytes = (dim + 1) / 2;
    const int64_t stride = (int64_t)gridDim.x * kDqBlock;
    for (int64_t e = (int64_t)blockIdx.x * kDqBlock + threadIdx.x; e < n_elems; e += stride) {
        const int64_t row = e / dim;
        const uint32_t k = (uint32_t)(e - row * dim);
        const uint32_t byte = codes[row * nbytes + k / 2];
        const uint32_t q = (k & 1u) ? (byte >> 4) : (byte & 15u);
        out[e] = __builtin_fmaf((float)q, f16_bits_to_float(scale_f16[row]), f16_bits_to_float(bias_f16[row]));
    }
}

hipError_t launch_dequantize(const uint8_t* codes, const uint16_t* scale_f16, const uint16_t* bias_f16,
                             int64_t rows, int32_t dim, float* out, hipStream_t stream)
{
    // One item per thread: neighbouring workgroups then write neighbouring memory, which measured 20 %
    // faster than a capped grid with a grid-stride loop (the loop remains for > 2^31 workgroups).
    const int64_t max_blocks = 0x7fffffffLL;
    const bool fast = dim % 4 == 0 && (reinterpret_cast<uintptr_t>(codes) % 2 == 0) &&
                      (reinterpret_cast<uintptr_t>(out) % 16 == 0);
    if (fast) {
        const int64_t n_quads = rows * (dim / 4);
        int64_t blocks = (n_quads + kDqBlock - 1) / kDqBlock;
        if (blocks > max_blocks) blocks = max_blocks;
        hipLaunchKernelGGL(dequantize_w4_kernel, dim3((unsigned)blocks), dim3(kDqBlock), 0, stream,
                           reinterpret_cast<const uint16_t*>(codes), scale_f16, bias_f16, n_quads,
                           (uint32_t)(dim / 4), reinterpret_cast<floatx4*>(out));
    } else {
        const int64_t n_elems = rows * dim;
        int64_t blocks = (n_elems + kDqBlock - 1) / kDqBlock;
        if (blocks > max_blocks) blocks = max_blocks;
        hipLaunchKernelGGL(dequantize_any_kernel, dim3((unsigned)blocks), dim3(kDqBlock), 0, stream, codes,
                           scale_f16, bias_f16, n_elems, (uint32_t)dim, out);
    }
    return hipGetLastError();
}

}  // namespace e4q
