// Issue rates of the instructions the score kernel is made of, measured on the GPU at hand (gfx950).
//
// A measurement aid like the streaming probe of gen.hip: no scoring arithmetic, no memory traffic beyond one result
// store per thread.  Every workgroup is 256 threads, i.e. one wave on each SIMD of its CU; 256 * W workgroups that
// each claim 1/W of a CU's LDS put W waves on every SIMD.  A wave runs a long loop of one instruction pattern on
// independent registers; the figure reported is the time per instruction and SIMD, in ns and in shader clocks
// (s_memtime ticks at the shader clock, s_memrealtime at 100 MHz).  Build: hipcc --offload-arch=gfx950 -O2.
#include <hip/hip_runtime.h>

#include <cstdio>

typedef float float4v __attribute__((ext_vector_type(4)));

#define REP4(x) x x x x
#define VA "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)
#define EIGHT(op, tail)                                                                                              \
    REP4(op " %0, " tail "\n " op " %1, " tail "\n " op " %2, " tail "\n " op " %3, " tail "\n " op " %4, " tail      \
            "\n " op " %5, " tail "\n " op " %6, " tail "\n " op " %7, " tail "\n ")

enum Op {
    kAdd, kMulFma, kAndShift, kFmacSgpr, kDot2, kAlignbit, kSqrt, kPermlane32, kAddDpp, kFmaF64, kMfma4x4x1,
    kMfma4x4x4f16, kMfmaThenValu, kMfmaBetweenValu, kBpermute, kDsRead128, kOps
};

template <int OP>
__global__ __launch_bounds__(256) void probe_kernel(float *out, int iters, long long *clk)
{
    extern __shared__ float lds[];
    const int tid = threadIdx.x;
    float a0 = tid * 1e-3f, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, a4 = a0 + 4, a5 = a0 + 5, a6 = a0 + 6, a7 = a0 + 7;
    const float b = 1.0001f, c = 0.5f;
    const float sb = __builtin_amdgcn_readfirstlane(b);
    const unsigned u0 = tid * 2654435761u, u1 = u0 ^ 0x12345u;
    double d0 = a0, d1 = a1, d2 = a2, d3 = a3;
    const double db = b;
    float4v m0 = {0, 0, 0, 0}, m1 = m0, m2 = m0, m3 = m0;
    const int lane_addr = (tid & 63) * 4, row_addr = (tid & 63) * 16;
    lds[tid] = a0;
    __syncthreads();
    const long long t0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        if constexpr (OP == kAdd) asm volatile(EIGHT("v_add_f32", "%8, %9") : VA : "v"(b), "v"(c));
        if constexpr (OP == kMulFma)
            asm volatile(REP4("v_mul_f32 %0, %8, %9\n v_fma_f32 %1, %8, %9, %0\n v_mul_f32 %2, %8, %9\n v_fma_f32 %3, %8, %9, %2\n"
                              "v_mul_f32 %4, %8, %9\n v_fma_f32 %5, %8, %9, %4\n v_mul_f32 %6, %8, %9\n v_fma_f32 %7, %8, %9, %6\n")
                         : VA : "v"(b), "v"(c));
        if constexpr (OP == kAndShift)
            asm volatile(REP4("v_and_b32 %0, 0xffff0000, %8\n v_lshlrev_b32 %1, 16, %8\n v_and_b32 %2, 0xffff0000, %8\n"
                              "v_lshlrev_b32 %3, 16, %8\n v_and_b32 %4, 0xffff0000, %8\n v_lshlrev_b32 %5, 16, %8\n"
                              "v_and_b32 %6, 0xffff0000, %8\n v_lshlrev_b32 %7, 16, %8\n")
                         : VA : "v"(u0));
        if constexpr (OP == kFmacSgpr) asm volatile(EIGHT("v_fmac_f32", "%8, %9") : VA : "s"(sb), "v"(c));
        if constexpr (OP == kDot2) asm volatile(EIGHT("v_dot2_f32_bf16", "%8, %9, 0") : VA : "v"(u0), "v"(u1));
        if constexpr (OP == kAlignbit) asm volatile(EIGHT("v_alignbit_b32", "%8, %8, 16") : VA : "v"(u0));
        if constexpr (OP == kSqrt) asm volatile(EIGHT("v_sqrt_f32", "%8") : VA : "v"(b));
        if constexpr (OP == kPermlane32)
            asm volatile(REP4("v_permlane32_swap_b32 %0, %1\n v_permlane32_swap_b32 %2, %3\n v_permlane32_swap_b32 %4, %5\n"
                              "v_permlane32_swap_b32 %6, %7\n v_permlane32_swap_b32 %0, %1\n v_permlane32_swap_b32 %2, %3\n"
                              "v_permlane32_swap_b32 %4, %5\n v_permlane32_swap_b32 %6, %7\n")
                         : VA);
        if constexpr (OP == kAddDpp)
            asm volatile(EIGHT("v_add_f32_dpp", "%8, %8 row_ror:8 row_mask:0xf bank_mask:0xf") : VA : "v"(b));
        if constexpr (OP == kFmaF64)
            asm volatile(REP4("v_fma_f64 %0, %4, %4, %0\n v_fma_f64 %1, %4, %4, %1\n v_fma_f64 %2, %4, %4, %2\n v_fma_f64 %3, %4, %4, %3\n"
                              "v_fma_f64 %0, %4, %4, %0\n v_fma_f64 %1, %4, %4, %1\n v_fma_f64 %2, %4, %4, %2\n v_fma_f64 %3, %4, %4, %3\n")
                         : "+v"(d0), "+v"(d1), "+v"(d2), "+v"(d3) : "v"(db));
        if constexpr (OP == kMfma4x4x1)   // four accumulators in turn
            asm volatile(REP4("v_mfma_f32_4x4x1_16b_f32 %0, %4, %5, %0\n v_mfma_f32_4x4x1_16b_f32 %1, %4, %5, %1\n"
                              "v_mfma_f32_4x4x1_16b_f32 %2, %4, %5, %2\n v_mfma_f32_4x4x1_16b_f32 %3, %4, %5, %3\n"
                              "v_mfma_f32_4x4x1_16b_f32 %0, %4, %5, %0\n v_mfma_f32_4x4x1_16b_f32 %1, %4, %5, %1\n"
                              "v_mfma_f32_4x4x1_16b_f32 %2, %4, %5, %2\n v_mfma_f32_4x4x1_16b_f32 %3, %4, %5, %3\n")
                         : "+v"(m0), "+v"(m1), "+v"(m2), "+v"(m3) : "v"(b), "v"(c));
        if constexpr (OP == kMfma4x4x4f16)
            asm volatile(REP4("v_mfma_f32_4x4x4_16b_f16 %0, %4, %4, %0\n v_mfma_f32_4x4x4_16b_f16 %1, %4, %4, %1\n"
                              "v_mfma_f32_4x4x4_16b_f16 %2, %4, %4, %2\n v_mfma_f32_4x4x4_16b_f16 %3, %4, %4, %3\n"
                              "v_mfma_f32_4x4x4_16b_f16 %0, %4, %4, %0\n v_mfma_f32_4x4x4_16b_f16 %1, %4, %4, %1\n"
                              "v_mfma_f32_4x4x4_16b_f16 %2, %4, %4, %2\n v_mfma_f32_4x4x4_16b_f16 %3, %4, %4, %3\n")
                         : "+v"(m0), "+v"(m1), "+v"(m2), "+v"(m3) : "v"(db));
        if constexpr (OP == kMfmaThenValu) {   // 16 matrix instructions in one run, then 32 additions
            asm volatile(REP4("v_mfma_f32_4x4x1_16b_f32 %0, %2, %3, %0\n v_mfma_f32_4x4x1_16b_f32 %1, %2, %3, %1\n"
                              "v_mfma_f32_4x4x1_16b_f32 %0, %2, %3, %0\n v_mfma_f32_4x4x1_16b_f32 %1, %2, %3, %1\n")
                         : "+v"(m0), "+v"(m1) : "v"(b), "v"(c));
            asm volatile(EIGHT("v_add_f32", "%8, %9") : VA : "v"(b), "v"(c));
        }
        if constexpr (OP == kMfmaBetweenValu)   // the same 16 + 32, one matrix instruction after every two additions
            asm volatile(REP4("v_mfma_f32_4x4x1_16b_f32 %0, %5, %6, %0\n v_add_f32 %2, %2, %5\n v_add_f32 %3, %3, %5\n"
                              "v_mfma_f32_4x4x1_16b_f32 %1, %5, %6, %1\n v_add_f32 %4, %4, %5\n v_add_f32 %2, %2, %5\n"
                              "v_mfma_f32_4x4x1_16b_f32 %0, %5, %6, %0\n v_add_f32 %3, %3, %5\n v_add_f32 %4, %4, %5\n"
                              "v_mfma_f32_4x4x1_16b_f32 %1, %5, %6, %1\n v_add_f32 %2, %2, %5\n v_add_f32 %3, %3, %5\n")
                         : "+v"(m0), "+v"(m1), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(b), "v"(c));
        if constexpr (OP == kBpermute)
            asm volatile(REP4("ds_bpermute_b32 %0, %8, %9\n ds_bpermute_b32 %1, %8, %9\n ds_bpermute_b32 %2, %8, %9\n"
                              "ds_bpermute_b32 %3, %8, %9\n ds_bpermute_b32 %4, %8, %9\n ds_bpermute_b32 %5, %8, %9\n"
                              "ds_bpermute_b32 %6, %8, %9\n ds_bpermute_b32 %7, %8, %9\n s_waitcnt lgkmcnt(0)\n")
                         : VA : "v"(lane_addr), "v"(b));
        if constexpr (OP == kDsRead128)   // 16 consecutive bytes per lane: no bank conflicts
            asm volatile(REP4("ds_read_b128 %0, %4\n ds_read_b128 %1, %4 offset:1024\n ds_read_b128 %2, %4 offset:2048\n"
                              "ds_read_b128 %3, %4 offset:3072\n ds_read_b128 %0, %4 offset:4096\n ds_read_b128 %1, %4 offset:5120\n"
                              "ds_read_b128 %2, %4 offset:6144\n ds_read_b128 %3, %4 offset:7168\n s_waitcnt lgkmcnt(0)\n")
                         : "+v"(m0), "+v"(m1), "+v"(m2), "+v"(m3) : "v"(row_addr));
    }
    const long long t1 = clock64(), w1 = wall_clock64();
    out[blockIdx.x * 256 + tid] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7 + m0[0] + m1[1] + m2[2] + m3[3] + (float)(d0 + d1 + d2 + d3);
    if (blockIdx.x == 0 && tid == 0) {
        clk[0] = t1 - t0;
        clk[1] = w1 - w0;
    }
}

template <int OP>
static int run(const char *name, int inst_per_iter, int waves_per_simd, float *out, long long *clk)
{
    const int iters = 20000;
    const int lds = waves_per_simd == 1 ? 120 * 1024 : waves_per_simd == 2 ? 70 * 1024 : 36 * 1024;
    if (hipFuncSetAttribute((const void *)probe_kernel<OP>, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return 1;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
    int n_cu = 0;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, 0) != hipSuccess) return 1;
    const int grid = n_cu * waves_per_simd;
    hipLaunchKernelGGL(probe_kernel<OP>, dim3(grid), dim3(256), lds, 0, out, 100, clk);
    (void)hipEventRecord(e0, 0);
    hipLaunchKernelGGL(probe_kernel<OP>, dim3(grid), dim3(256), lds, 0, out, iters, clk);
    (void)hipEventRecord(e1, 0);
    if (hipDeviceSynchronize() != hipSuccess) return 1;
    float ms = 0;
    (void)hipEventElapsedTime(&ms, e0, e1);
    long long h[2];
    if (hipMemcpy(h, clk, sizeof h, hipMemcpyDeviceToHost) != hipSuccess) return 1;
    const double per_simd = (double)iters * inst_per_iter * waves_per_simd;
    const double ghz = (double)h[0] / ((double)h[1] * 10.0);
    const double ns = ms * 1e6 / per_simd;
    printf("| %-52s | %d | %7.3f | %6.2f | %5.2f |\n", name, waves_per_simd, ns, ns * ghz, ghz);
    fflush(stdout);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return 0;
}

int main()
{
    float *out = nullptr;
    long long *clk = nullptr;
    if (hipMalloc(&out, (size_t)1024 * 4 * 256 * sizeof(float)) != hipSuccess || hipMalloc(&clk, 16) != hipSuccess) return 1;
    printf("| instruction pattern (per instruction unless noted) | waves per SIMD | ns per SIMD | shader clocks | GHz |\n|---|---|---|---|---|\n");
    int rc = 0;
    for (int w : {1, 4}) {
        rc |= run<kAdd>("v_add_f32", 32, w, out, clk);
        rc |= run<kMulFma>("v_mul_f32 / v_fma_f32", 32, w, out, clk);
        rc |= run<kAndShift>("v_and_b32 / v_lshlrev_b32 (bf16 unpack)", 32, w, out, clk);
        rc |= run<kFmacSgpr>("v_fmac_f32 with a scalar-register operand", 32, w, out, clk);
        rc |= run<kDot2>("v_dot2_f32_bf16", 32, w, out, clk);
        rc |= run<kAlignbit>("v_alignbit_b32", 32, w, out, clk);
        rc |= run<kSqrt>("v_sqrt_f32", 32, w, out, clk);
        rc |= run<kPermlane32>("v_permlane32_swap_b32", 32, w, out, clk);
        rc |= run<kAddDpp>("v_add_f32_dpp row_ror", 32, w, out, clk);
        rc |= run<kFmaF64>("v_fma_f64", 32, w, out, clk);
        rc |= run<kMfma4x4x1>("v_mfma_f32_4x4x1_16b_f32", 32, w, out, clk);
        rc |= run<kMfma4x4x4f16>("v_mfma_f32_4x4x4_16b_f16", 32, w, out, clk);
        rc |= run<kMfmaThenValu>("16 x 4x4x1 in one run, then 32 v_add (per 48)", 1, w, out, clk);
        rc |= run<kMfmaBetweenValu>("16 x (4x4x1 + 2 v_add), alternating (per 48)", 1, w, out, clk);
        rc |= run<kBpermute>("ds_bpermute_b32", 32, w, out, clk);
        rc |= run<kDsRead128>("ds_read_b128", 32, w, out, clk);
    }
    return rc;
}
