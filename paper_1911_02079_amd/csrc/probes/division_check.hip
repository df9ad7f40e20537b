// Exhaustive check of the two short divisions of the greedy search (e4q_device.h: div_by_qmax, rcp_of_f16_value)
// against the compiler's correctly rounded division sequence, on the device they run on.
// Not part of libe4q; it backs the claim that the short forms change no result.
//
//   hipcc --offload-arch=gfx950 -O3 -ffp-contract=off -fhip-fp32-correctly-rounded-divide-sqrt -fno-fast-math \
//       -Xclang -target-feature -Xclang -packed-fp32-ops -I paper_1911_02079_amd/csrc \
//       paper_1911_02079_amd/csrc/probes/division_check.hip -o division_check && ./division_check
//
// x / qmax: all 2^32 binary32 bit patterns of x (NaN and infinity skipped) for qmax = 3, 15, 255 (2, 4 and 8 bits).
// 1 / s: all 65 536 binary16 bit patterns of s (NaN, infinity and zero skipped).
// Exit status 0 when the only difference is x = -0 (the short form returns +0; a range hi - lo is never -0).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>

#include "e4q_device.h"

#define CK(x)                                                                      \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 2;                                                              \
        }                                                                          \
    } while (0)

// counts[0]: binary32 results that differ, x = -0 aside; counts[1]: x = -0 differs; first: smallest |x| bits that differ
__global__ void __launch_bounds__(256) check_div_by_qmax(float qmax, float rq, unsigned long long* counts, uint32_t* first)
{
    unsigned long long bad = 0, bad_negzero = 0;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < (1ull << 32); i += stride) {
        const uint32_t bits = (uint32_t)i;
        const float x = __builtin_bit_cast(float, bits);
        if (!(x == x) || __builtin_isinf(x)) continue;
        const float want = x / qmax;
        const float got = e4q::div_by_qmax(x, qmax, rq);
        if (__builtin_bit_cast(uint32_t, want) != __builtin_bit_cast(uint32_t, got)) {
            if (bits == 0x80000000u) {
                ++bad_negzero;
            } else {
                ++bad;
                atomicMin(first, bits & 0x7fffffffu);
            }
        }
    }
    if (bad) atomicAdd(&counts[0], bad);
    if (bad_negzero) atomicAdd(&counts[1], bad_negzero);
}

__global__ void __launch_bounds__(256) check_rcp_of_f16_value(unsigned long long* counts, uint32_t* first)
{
    const uint32_t h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= 65536u) return;
    const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)h);
    if (!(s == s) || __builtin_isinf(s) || s == 0.0f) return;
    const float want = 1.0f / s, got = e4q::rcp_of_f16_value(s);
    if (__builtin_bit_cast(uint32_t, want) != __builtin_bit_cast(uint32_t, got)) {
        atomicAdd(&counts[0], 1ull);
        atomicMin(first, h);
    }
}

int main()
{
    unsigned long long* counts;
    uint32_t* first;
    CK(hipMalloc(&counts, 16));
    CK(hipMalloc(&first, 4));
    unsigned long long h[2];
    uint32_t f;
    bool ok = true;
    const float qmaxes[3] = {3.0f, 15.0f, 255.0f};
    for (float qmax : qmaxes) {
        CK(hipMemset(counts, 0, 16));
        CK(hipMemset(first, 0xff, 4));
        hipLaunchKernelGGL(check_div_by_qmax, dim3(8192), dim3(256), 0, 0, qmax, 1.0f / qmax, counts, first);
        CK(hipGetLastError());
        CK(hipDeviceSynchronize());
        CK(hipMemcpy(h, counts, 16, hipMemcpyDeviceToHost));
        CK(hipMemcpy(&f, first, 4, hipMemcpyDeviceToHost));
        std::printf("x / %g over all finite binary32 x: %llu results differ (smallest |x| bits 0x%08x), x = -0 differs: %llu\n",
                    qmax, h[0], f, h[1]);
        ok = ok && h[0] == 0;
    }
    CK(hipMemset(counts, 0, 16));
    CK(hipMemset(first, 0xff, 4));
    hipLaunchKernelGGL(check_rcp_of_f16_value, dim3(256), dim3(256), 0, 0, counts, first);
    CK(hipGetLastError());
    CK(hipDeviceSynchronize());
    CK(hipMemcpy(h, counts, 16, hipMemcpyDeviceToHost));
    CK(hipMemcpy(&f, first, 4, hipMemcpyDeviceToHost));
    std::printf("1 / s over all finite non-zero binary16 s: %llu results differ (first bits 0x%04x)\n", h[0], f);
    ok = ok && h[0] == 0;
    CK(hipFree(counts));
    CK(hipFree(first));
    std::printf(ok ? "PASS\n" : "FAIL\n");
    return ok ? 0 : 1;
}
