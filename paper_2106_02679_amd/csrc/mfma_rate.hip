// Calibration: the bf16 MFMA rate the chip sustains on register operands alone - no memory, no LDS, nothing but
// v_mfma_f32_16x16x32_bf16 on every SIMD, in the issue order of the GEMM kernel's main loop: two products in a row on
// each accumulator.  With constant operands this reaches the nominal peak; with random mantissas and signs the chip's
// power management holds the clock lower, and that rate - not the nominal one - is what a GEMM on real activations
// can approach.  (The order matters at the power limit: with every instruction on another accumulator the same
// instruction runs about 8 % slower.)  Used by the benchmark tools only.
#include "kernels.h"
#include "../../include/lga_ops.h"

namespace lga {
namespace {

// CONSTANT: every operand value is 1.0; else values in [0.5, 1) with random sign and mantissa bits.
template <bool CONSTANT>
__global__ __launch_bounds__(256, 1) void mfma_rate_kernel(float *sink, int iters) {
    bf16x8 a[4], b[4];
    unsigned s = (threadIdx.x + 1) * 2654435761u ^ (blockIdx.x * 40503u);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        u32x4 va, vb;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            s = s * 1664525u + 1013904223u;
            const unsigned x = s;
            s = s * 1664525u + 1013904223u;
            const unsigned y = s;
            va[j] = CONSTANT ? 0x3f803f80u : ((x & 0x807f807fu) | 0x3f003f00u);      // two bf16 values per word
            vb[j] = CONSTANT ? 0x3f803f80u : ((y & 0x807f807fu) | 0x3f003f00u);
        }
        a[i] = __builtin_bit_cast(bf16x8, va);
        b[i] = __builtin_bit_cast(bf16x8, vb);
    }
    f32x4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                mfma_16x16x32_acc<bf16>(a[i], b[j], acc[i * 4 + j]);
                mfma_16x16x32_acc<bf16>(a[i ^ 1], b[j ^ 1], acc[i * 4 + j]);
                __builtin_amdgcn_sched_barrier(0);
            }
    }
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");      // see mfma_16x16x32_acc
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) t += acc[i][r];
    sink[blockIdx.x * 256 + threadIdx.x] = t;
}

}  // namespace
}  // namespace lga

extern "C" int lga_op_mfma_rate(int32_t iters, int32_t mode, float *sink, double *tflops, void *stream) {
    using namespace lga;
    if (iters < 1 || iters > (1 << 23) || mode < 0 || mode > 1 || !sink || !tflops) return LGA_ERR_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return LGA_ERR_HIP;
    if (cus < 1 || cus > 256) cus = 256;                    // sink holds 256 workgroups' results
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return LGA_ERR_HIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return LGA_ERR_HIP;
    }
    (void)hipEventRecord(e0, s);
    if (mode == 0) hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(cus), dim3(256), 0, s, sink, iters);
    else hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(cus), dim3(256), 0, s, sink, iters);
    (void)hipEventRecord(e1, s);
    hipError_t e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess || hipGetLastError() != hipSuccess) return LGA_ERR_HIP;
    // per workgroup: 4 wavefronts x iters x 32 MFMAs of 16 x 16 x 32 x 2 flop
    *tflops = (double)cus * 4.0 * iters * 32.0 * 16384.0 / (ms * 1e9);
    return LGA_OK;
}
