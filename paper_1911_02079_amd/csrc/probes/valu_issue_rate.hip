// Issue-rate probe for gfx950: how often one SIMD issues a wave64 vector instruction of a given kind.
// Not part of libe4q; it backs the instruction-rate table the kernels' rooflines and layouts are argued from.
//
//   hipcc --offload-arch=gfx950 -O2 -Xclang -target-feature -Xclang -packed-fp32-ops \
//       paper_1911_02079_amd/csrc/probes/valu_issue_rate.hip -o valu_issue_rate && ./valu_issue_rate
//
// Every kernel runs ITER x 16 copies of a body on one wave per workgroup, w workgroups per SIMD (w = 1, 2, 3, 4, 8);
// a body is 9 copies of one instruction on 9 independent registers, or one of the compare / select patterns of the
// codebook kernel's bisection.  Prints cycles (at the 2.4 GHz the peak is quoted at) per instruction per SIMD.
// All kernels terminate after a fixed trip count and touch no memory except one guarded store.
#include <hip/hip_runtime.h>

#include <cstdio>

#define CK(x)                                                                      \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                              \
        }                                                                          \
    } while (0)

constexpr int ITER = 400;
#define R4(X) X X X X
#define R16(X) R4(X) R4(X) R4(X) R4(X)
// registers a0..a8 (%0..%8), b (%9), c (%10), x (%11); VCC and s[20:23] hold conditions set before the loop
#define KERNEL(NAME, BODY)                                                                                          \
    __global__ void __launch_bounds__(64) NAME(float* out, float b, float c)                                        \
    {                                                                                                               \
        float a0 = threadIdx.x, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, a4 = a0 + 4, a5 = a0 + 5, a6 = a0 + 6,        \
              a7 = a0 + 7, a8 = a0 + 8;                                                                             \
        float x = b * threadIdx.x;                                                                                  \
        asm volatile("v_cmp_lt_f32 vcc, %0, %1\n v_cmp_lt_f32 s[20:21], %0, %1\n v_cmp_gt_f32 s[22:23], %0, %1\n s_nop 4" \
                     :: "v"(x), "v"(c) : "vcc", "s20", "s21", "s22", "s23");                                        \
        for (int it = 0; it < ITER; ++it) {                                                                         \
            R16(BODY)                                                                                               \
        }                                                                                                           \
        float s = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7 + a8;                                                       \
        if (s == 12345.0f) out[threadIdx.x] = s;                                                                    \
    }
#define REGS : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7), "+v"(a8) : "v"(b), "v"(c), "v"(x)
#define NINE(I, TAIL) I " %0, " TAIL("%0") "\n" I " %1, " TAIL("%1") "\n" I " %2, " TAIL("%2") "\n" I " %3, " TAIL("%3") "\n" \
                      I " %4, " TAIL("%4") "\n" I " %5, " TAIL("%5") "\n" I " %6, " TAIL("%6") "\n" I " %7, " TAIL("%7") "\n" \
                      I " %8, " TAIL("%8") "\n"
#define T_B_SELF(R) "%9, " R              /* op d, b, d */
#define T_B_SELF_C(R) "%9, " R ", %10"    /* op d, b, d, c */
#define T_SELF(R) R                       /* op d, d */
#define T_SEL_VCC(R) "%9, " R ", vcc"
#define T_SEL_S20(R) "%9, " R ", s[20:21]"
#define T_SEL_S22(R) "%9, " R ", s[22:23]"
#define T_SHL_ADD(R) R ", 3, %9"
#define T_SGPR(R) "s20, " R
#define T_MED3_K(R) R ", %9, 0"

KERNEL(k_add, asm volatile(NINE("v_add_f32_e32", T_B_SELF) REGS);)
KERNEL(k_mul, asm volatile(NINE("v_mul_f32_e32", T_B_SELF) REGS);)
KERNEL(k_fma, asm volatile(NINE("v_fma_f32", T_B_SELF_C) REGS);)
KERNEL(k_mov, asm volatile(NINE("v_mov_b32_e32", T_SELF) REGS);)
KERNEL(k_add_sgpr, asm volatile(NINE("v_add_f32_e32", T_SGPR) REGS : "s20");)
KERNEL(k_rndne, asm volatile(NINE("v_rndne_f32_e32", T_SELF) REGS);)
KERNEL(k_med3, asm volatile(NINE("v_med3_f32", T_MED3_K) REGS);)
KERNEL(k_min3, asm volatile(NINE("v_min3_f32", T_B_SELF_C) REGS);)
KERNEL(k_min, asm volatile(NINE("v_min_f32_e32", T_B_SELF) REGS);)
KERNEL(k_cvt_f16, asm volatile(NINE("v_cvt_f16_f32_e32", T_SELF) REGS);)
KERNEL(k_add_u32, asm volatile(NINE("v_add_u32_e32", T_B_SELF) REGS);)
KERNEL(k_lshl_add, asm volatile(NINE("v_lshl_add_u32", T_SHL_ADD) REGS);)
KERNEL(k_or3, asm volatile(NINE("v_or3_b32", T_B_SELF_C) REGS);)
KERNEL(k_cmp, asm volatile("v_cmp_ge_f32_e32 vcc, %11, %0\n v_cmp_ge_f32_e32 vcc, %11, %1\n v_cmp_ge_f32_e32 vcc, %11, %2\n"
                           "v_cmp_ge_f32_e32 vcc, %11, %3\n v_cmp_ge_f32_e32 vcc, %11, %4\n v_cmp_ge_f32_e32 vcc, %11, %5\n"
                           "v_cmp_ge_f32_e32 vcc, %11, %6\n v_cmp_ge_f32_e32 vcc, %11, %7\n v_cmp_ge_f32_e32 vcc, %11, %8\n" REGS : "vcc");)
// selects: on VCC written before the loop; on a scalar register pair; right behind their compare; ten instructions behind it
KERNEL(k_sel_vcc_stale, asm volatile(NINE("v_cndmask_b32_e32", T_SEL_VCC) REGS : "vcc");)
KERNEL(k_sel_pair, asm volatile(NINE("v_cndmask_b32_e64", T_SEL_S20) REGS : "s20", "s21");)
KERNEL(k_cmp_sel_vcc, asm volatile("v_cmp_ge_f32_e32 vcc, %11, %0\n s_nop 1\n" NINE("v_cndmask_b32_e32", T_SEL_VCC) REGS : "vcc");)
KERNEL(k_cmp_sel_pair, asm volatile("v_cmp_ge_f32_e64 s[20:21], %11, %0\n s_nop 1\n" NINE("v_cndmask_b32_e64", T_SEL_S20) REGS : "s20", "s21");)
KERNEL(k_cmp_9add_sel_vcc, asm volatile("v_cmp_ge_f32_e32 vcc, %11, %0\n" NINE("v_add_f32_e32", T_B_SELF) NINE("v_cndmask_b32_e32", T_SEL_VCC) REGS : "vcc");)
KERNEL(k_2cmp_sel_pairs, asm volatile("v_cmp_ge_f32_e64 s[20:21], %11, %0\n v_cmp_ge_f32_e64 s[22:23], %11, %1\n"
                                      NINE("v_cndmask_b32_e64", T_SEL_S20) NINE("v_cndmask_b32_e64", T_SEL_S22) REGS : "s20", "s21", "s22", "s23");)
// the greedy search's eight operations per element and range, on three of the registers
KERNEL(k_greedy_mix, asm volatile(
    "v_sub_f32_e32 %0, %0, %9\n v_sub_f32_e32 %1, %1, %9\n v_sub_f32_e32 %2, %2, %9\n"
    "v_mul_f32_e32 %0, %10, %0\n v_mul_f32_e32 %1, %10, %1\n v_mul_f32_e32 %2, %10, %2\n"
    "v_rndne_f32_e32 %0, %0\n v_rndne_f32_e32 %1, %1\n v_rndne_f32_e32 %2, %2\n"
    "v_med3_f32 %0, %0, %9, 0\n v_med3_f32 %1, %1, %9, 0\n v_med3_f32 %2, %2, %9, 0\n"
    "v_fma_f32 %0, %0, %9, %10\n v_fma_f32 %1, %1, %9, %10\n v_fma_f32 %2, %2, %9, %10\n"
    "v_sub_f32_e32 %0, %0, %9\n v_sub_f32_e32 %1, %1, %9\n v_sub_f32_e32 %2, %2, %9\n"
    "v_mul_f32_e32 %0, %0, %0\n v_mul_f32_e32 %1, %1, %1\n v_mul_f32_e32 %2, %2, %2\n"
    "v_add_f32_e32 %0, %0, %10\n v_add_f32_e32 %1, %1, %10\n v_add_f32_e32 %2, %2, %10\n" REGS);)

__global__ void __launch_bounds__(64) k_f64(double* out, double b, double c)
{
    double a0 = threadIdx.x, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, a4 = a0 + 4, a5 = a0 + 5, a6 = a0 + 6, a7 = a0 + 7, a8 = a0 + 8;
    for (int it = 0; it < ITER; ++it) {
        R16(asm volatile(NINE("v_fma_f64", T_B_SELF_C) : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7), "+v"(a8) : "v"(b), "v"(c));)
    }
    double s = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7 + a8;
    if (s == 12345.0) out[threadIdx.x] = s;
}

template <typename T, typename K>
int run(const char* name, K kern, int instr_per_body, int waves_per_simd)
{
    T* out;
    CK(hipMalloc(&out, 64 * sizeof(T)));
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int blocks = prop.multiProcessorCount * 4 * waves_per_simd;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(64), 0, 0, out, (T)1, (T)2);
    CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int rep = 0; rep < 5; ++rep) {
        CK(hipEventRecord(e0, 0));
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(64), 0, 0, out, (T)1, (T)2);
        CK(hipEventRecord(e1, 0));
        CK(hipEventSynchronize(e1));
        float ms;
        CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    const double instr = (double)waves_per_simd * ITER * 16 * instr_per_body;
    std::printf("%-22s %d waves/SIMD  %8.3f ms  %6.2f cycles per instruction\n", name, waves_per_simd, best, best * 1e-3 * 2.4e9 / instr);
    std::fflush(stdout);
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    CK(hipFree(out));
    return 0;
}

int main()
{
    for (int w : {1, 2, 3, 4, 8}) {
#define RUN(NAME, KERN, N) if (run<float>(NAME, KERN, N, w)) return 1;
        RUN("v_add_f32", k_add, 9) RUN("v_mul_f32", k_mul, 9) RUN("v_fma_f32", k_fma, 9) RUN("v_mov_b32", k_mov, 9)
        RUN("v_add_f32 (SGPR src)", k_add_sgpr, 9) RUN("v_rndne_f32", k_rndne, 9) RUN("v_med3_f32", k_med3, 9)
        RUN("v_min3_f32", k_min3, 9) RUN("v_min_f32", k_min, 9) RUN("v_cvt_f16_f32", k_cvt_f16, 9)
        RUN("v_add_u32", k_add_u32, 9) RUN("v_lshl_add_u32", k_lshl_add, 9) RUN("v_or3_b32", k_or3, 9)
        RUN("v_cmp_ge_f32", k_cmp, 9) RUN("select, stale VCC", k_sel_vcc_stale, 9) RUN("select, SGPR pair", k_sel_pair, 9)
        RUN("cmp; 9 sel VCC", k_cmp_sel_vcc, 10) RUN("cmp; 9 sel pair", k_cmp_sel_pair, 10)
        RUN("cmp; 9 add; 9 sel VCC", k_cmp_9add_sel_vcc, 19) RUN("2 cmp; 18 sel pairs", k_2cmp_sel_pairs, 20)
        RUN("greedy mix (6 + 2)", k_greedy_mix, 24)
#undef RUN
        if (run<double>("v_fma_f64", k_f64, 9, w)) return 1;
    }
    return 0;
}
