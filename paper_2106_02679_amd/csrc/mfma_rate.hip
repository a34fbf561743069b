// Calibration: the bf16 MFMA rate the chip sustains on register operands alone - no memory, no LDS, nothing but
// v_mfma_f32_32x32x16_bf16 back to back on every SIMD.  With constant operands this reaches the nominal peak; with
// random mantissas and signs the chip's power management holds the clock lower, and that rate - not the
// nominal one - is what a GEMM on real activations can approach.  A third mode re-reads the operands from LDS the
// way a 2 x 2-wavefront 256 x 256 GEMM tile must (eight 16-byte reads per 16 MFMAs, issued 16 MFMAs ahead): what is
// left once the operands have to come from somewhere.  Modes 3 and 4 add what fills LDS in a GEMM - direct-to-LDS
// loads of 64 KB per 64 MFMAs of each wavefront, from a 4 MB window that stays in L2 - and the barrier per k tile:
// together the structural ceiling of an output-stationary 256 x 256 tile kernel on this chip, before a byte has
// come from HBM.  Mode 5 is mode 0 with v_mfma_f32_32x32x16_f16 on IEEE half operands, whose three more mantissa bits
// toggle too.  Used by the benchmark tools only.
#include <cstdio>

#include "kernels.h"
#include "../../include/lga_ops.h"

namespace lga {
namespace {

constexpr int kLdsChunks = 8192;        // 128 KB of operand data in LDS (mode 2)

// mode 0: random register operands; 1: constant register operands; 2: random operands re-read from LDS;
// 3: as 2, plus direct-to-LDS loads at a GEMM tile's rate; 4: as 3, plus a barrier per k tile;
// 5: random register operands in IEEE half, the f16 instruction;
// 6: register operands (as 0) plus the direct-to-LDS loads of 3, nothing reads LDS; 7: register operands plus the same
// bytes loaded into registers instead of LDS (taken apart: what of mode 3's loss is the way from L2 to the CU, what
// is LDS); 8: register operands plus the same bytes loaded into registers and written to LDS with ds_write_b128 three
// MFMA groups later (the classic staging, against 6); 9: as 0 with v_mfma_f32_16x16x32_bf16 (twice as many instructions
// for the same flops, half the operand reuse per instruction); 10: as 7 with twice the bytes (128 KB per k tile and CU:
// what a kernel would move if every wavefront fetched its own operands into registers, with no LDS and no barrier)
typedef __attribute__((address_space(3))) void *lds_ptr_t;
constexpr int kDmaWindow = 4 << 20;       // bytes of source data the loads of modes 3 and 4 walk over (L2-resident)

template <int MODE>
__global__ __launch_bounds__(256, 1) void mfma_rate_kernel(float *sink, const unsigned *src, int iters) {
    constexpr int constant_operands = MODE == 1;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4 *lds = reinterpret_cast<u32x4 *>(smem);
    // operand registers: values around +-1 with random mantissas and signs, or all ones
    bf16x8 a[4], b[4];
    unsigned s = (threadIdx.x + 1) * 2654435761u ^ (blockIdx.x * 40503u);
    if constexpr (MODE >= 2 && MODE <= 4) {
        for (int i = threadIdx.x; i < kLdsChunks; i += 256) {
            u32x4 v;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s = s * 1664525u + 1013904223u;
                v[j] = (s & 0x807f807fu) | 0x3f003f00u;
            }
            lds[i] = v;
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        u32x4 va, vb;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            s = s * 1664525u + 1013904223u;
            const unsigned x = s;
            s = s * 1664525u + 1013904223u;
            const unsigned y = s;
            // bf16: sign and 7 mantissa bits random, exponent of [0.5, 1); half: sign and 10 mantissa bits, same range
            va[j] = constant_operands ? 0x3f803f80u : MODE == 5 ? ((x & 0x83ff83ffu) | 0x38003800u) : ((x & 0x807f807fu) | 0x3f003f00u);
            vb[j] = constant_operands ? 0x3f803f80u : MODE == 5 ? ((y & 0x83ff83ffu) | 0x38003800u) : ((y & 0x807f807fu) | 0x3f003f00u);
        }
        a[i] = __builtin_bit_cast(bf16x8, va);
        b[i] = __builtin_bit_cast(bf16x8, vb);
    }
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    bf16x8 a2[4], b2[4];
    int off = threadIdx.x;
    // operand data lives in the first half of the 128 KB of LDS; modes 3 and 4 stream into the second half
    auto fetch = [&](bf16x8 (&fa)[4], bf16x8 (&fb)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[i] = __builtin_bit_cast(bf16x8, lds[(off + 256 * i) & (kLdsChunks / 2 - 1)]);
            fb[i] = __builtin_bit_cast(bf16x8, lds[(off + 256 * (i + 4) + 1024) & (kLdsChunks / 2 - 1)]);
        }
        off += 2048;
    };
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    u32x4 junk[4] = {}, junk2[4] = {};
    u32x4 stage[4][4] = {};          // mode 8: four sets of four 16-byte loads in flight
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned *>(src), 0, kDmaWindow, 0x00020000);
    unsigned goff = (blockIdx.x * 65536u + wave * 16384u) & (kDmaWindow - 1);
    for (int it = 0; it < iters; it += 4) {
        // one "k tile": four groups of 16 MFMAs; in modes >= 2 each group's operands are read while the previous group
        // runs; in modes >= 3 each wavefront also issues its 16 KB share of the tile's 64 KB of direct-to-LDS loads
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if constexpr (MODE == 8) {
                // write the set that was requested three groups ago (its loads are the oldest 4 of the 16 in flight), then
                // request into it again
                __builtin_amdgcn_s_waitcnt(0x0F70 | 12);        // vmcnt only
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<u32x4 *>(smem + kLdsChunks * 8 + wave * 16384 + (q * 4 + j) * 1024 + lane * 16) = stage[q][j];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    stage[q][j] = __builtin_amdgcn_raw_buffer_load_b128(
                        rs, (int)((goff + (q * 4 + j) * 1024 + lane * 16) & (kDmaWindow - 1)), 0, 0);
            }
            if constexpr (MODE == 10) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    junk2[j] = __builtin_amdgcn_raw_buffer_load_b128(
                        rs, (int)((goff + 32768u + (q * 4 + j) * 1024 + lane * 16) & (kDmaWindow - 1)), 0, 0);
            }
            if constexpr (MODE == 7 || MODE == 10) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    junk[j] = __builtin_amdgcn_raw_buffer_load_b128(
                        rs, (int)((goff + (q * 4 + j) * 1024 + lane * 16) & (kDmaWindow - 1)), 0, 0);
            }
            if constexpr (MODE == 3 || MODE == 4 || MODE == 6) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        rs, (lds_ptr_t)(smem + kLdsChunks * 8 + wave * 16384 + (q * 4 + j) * 1024), 16,
                        (int)((goff + (q * 4 + j) * 1024 + lane * 16) & (kDmaWindow - 1)), 0, 0, 0);
            }
            if constexpr (MODE >= 2 && MODE <= 4) {
                if (q & 1) fetch(a, b);
                else fetch(a2, b2);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    constexpr bool second = MODE >= 2 && MODE <= 4;       // operand sets alternate when they come from LDS
                    const bf16x8 fa = (second && (q & 1)) ? a2[i] : a[i], fb = (second && (q & 1)) ? b2[j] : b[j];
                    if constexpr (MODE == 9) {
                        f32x4 *a16 = reinterpret_cast<f32x4 *>(&acc[i * 4 + j]);
                        a16[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, a16[0], 0, 0, 0);
                        a16[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb, fa, a16[1], 0, 0, 0);
                    } else if constexpr (MODE == 5)
                        acc[i * 4 + j] = mfma_32x32x16<f16>(__builtin_bit_cast(x8<f16>, fa), __builtin_bit_cast(x8<f16>, fb),
                                                            acc[i * 4 + j]);
                    else
                        acc[i * 4 + j] = mfma_32x32x16<bf16>(fa, fb, acc[i * 4 + j]);
                }
        }
        goff = (goff + 65536u * 7u) & (kDmaWindow - 1);
        if constexpr (MODE == 3 || MODE == 4 || MODE == 6) __builtin_amdgcn_s_waitcnt(0x0070 | 15);
        if constexpr (MODE == 7 || MODE == 10) {            // keep the loaded values alive without touching the MFMAs
#pragma unroll
            for (int j = 0; j < 4; ++j) asm volatile("" ::"v"(junk[j]));
        }
        if constexpr (MODE == 10) {
#pragma unroll
            for (int j = 0; j < 4; ++j) asm volatile("" ::"v"(junk2[j]));
        }     // at most one tile's loads in flight
        if constexpr (MODE == 4) {
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) t += acc[i][r];
    sink[blockIdx.x * 256 + threadIdx.x] = t;
}

// Mode 11: a register-direct GEMM inner loop in miniature.  v_mfma_f32_16x16x32_bf16 on a 128 x 128 wavefront tile
// (8 x 8 blocks), both operands loaded straight from (L2-resident) memory into registers in the instruction's own
// layout - lane = (row l % 16, 16-byte k chunk l / 16), so the four lanes of a row read 64 contiguous bytes and one
// load instruction touches 16 rows - double-buffered one k step (32) ahead.  No LDS, no barrier; the four wavefronts
// of a workgroup form a 2 x 2 arrangement that shares row blocks only through the caches.  Rows are 4 KB + 128 B apart
// in a 2.1 MB window that every workgroup reads alike.
__global__ __launch_bounds__(256, 1) void mfma_direct_kernel(float *sink, const unsigned *src, int iters) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    constexpr int kRowBytes = 4096 + 128, kRowData = 4096;     // a pitch that is not a power of two
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned *>(src), 0, 4 << 20, 0x00020000);
    // rows 0..255: the A panel (wm selects a half), rows 256..511: the B panel (wn selects a half)
    const int offA = (wm * 128 + (lane & 15)) * kRowBytes + (lane >> 4) * 16;
    const int offB = (256 + wn * 128 + (lane & 15)) * kRowBytes + (lane >> 4) * 16;
    bf16x8 a[2][8], b[2][8];
    f32x4 acc[64];
#pragma unroll
    for (int i = 0; i < 64; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto fetch = [&](int buf, int kbyte) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[buf][i] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rs, offA + i * 16 * kRowBytes, kbyte, 0));
            b[buf][i] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(rs, offB + i * 16 * kRowBytes, kbyte, 0));
        }
    };
    int kbyte = 0;
    fetch(0, 0);
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {                         // two k steps of 32 = the flops of 64 32x32x16 MFMAs
            kbyte = (kbyte + 64) & (kRowData - 1);
            fetch(h ^ 1, kbyte);
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    acc[i * 8 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[h][j], a[h][i], acc[i * 8 + j], 0, 0, 0);
        }
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 64; ++i) t += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    sink[blockIdx.x * 256 + threadIdx.x] = t;
}

}  // namespace
}  // namespace lga

extern "C" int lga_op_mfma_rate(int32_t iters, int32_t mode, float *sink, double *tflops, void *stream) {
    using namespace lga;
    if (iters < 4 || iters > (1 << 24) || mode < 0 || mode > 11 || !sink || !tflops) return LGA_ERR_ARG;
    iters &= ~3;                                            // the loop does four groups of 16 MFMAs per turn
    // results go to the first 65536 floats of sink; modes 3 and 4 read the kDmaWindow bytes after them
    const unsigned *src = reinterpret_cast<const unsigned *>(sink + 65536);
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
    constexpr int kSmem = kLdsChunks * 16;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(mfma_rate_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, kSmem);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(mfma_rate_kernel<3>), hipFuncAttributeMaxDynamicSharedMemorySize, kSmem);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(mfma_rate_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, kSmem);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(mfma_rate_kernel<6>), hipFuncAttributeMaxDynamicSharedMemorySize, kSmem);
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(mfma_rate_kernel<8>), hipFuncAttributeMaxDynamicSharedMemorySize, kSmem);
        attr_set = true;
    }
    switch (mode) {
        case 0: hipLaunchKernelGGL(mfma_rate_kernel<0>, dim3(cus), dim3(256), 0, s, sink, src, iters); break;
        case 1: hipLaunchKernelGGL(mfma_rate_kernel<1>, dim3(cus), dim3(256), 0, s, sink, src, iters); break;
        case 2: hipLaunchKernelGGL(mfma_rate_kernel<2>, dim3(cus), dim3(256), kSmem, s, sink, src, iters); break;
        case 3: hipLaunchKernelGGL(mfma_rate_kernel<3>, dim3(cus), dim3(256), kSmem, s, sink, src, iters); break;
        case 4: hipLaunchKernelGGL(mfma_rate_kernel<4>, dim3(cus), dim3(256), kSmem, s, sink, src, iters); break;
        case 5: hipLaunchKernelGGL(mfma_rate_kernel<5>, dim3(cus), dim3(256), 0, s, sink, src, iters); break;
        case 6: hipLaunchKernelGGL(mfma_rate_kernel<6>, dim3(cus), dim3(256), kSmem, s, sink, src, iters); break;
        case 7: hipLaunchKernelGGL(mfma_rate_kernel<7>, dim3(cus), dim3(256), 0, s, sink, src, iters); break;
        case 8: hipLaunchKernelGGL(mfma_rate_kernel<8>, dim3(cus), dim3(256), kSmem, s, sink, src, iters); break;
        case 9: hipLaunchKernelGGL(mfma_rate_kernel<9>, dim3(cus), dim3(256), 0, s, sink, src, iters); break;
        case 10: hipLaunchKernelGGL(mfma_rate_kernel<10>, dim3(cus), dim3(256), 0, s, sink, src, iters); break;
        default: hipLaunchKernelGGL(mfma_direct_kernel, dim3(cus), dim3(256), 0, s, sink, src, iters); break;
    }
    (void)hipEventRecord(e1, s);
    hipError_t e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess || hipGetLastError() != hipSuccess) return LGA_ERR_HIP;
    // per workgroup: 4 wavefronts x iters x 16 MFMAs of 32 x 32 x 16 x 2 flop
    *tflops = (double)cus * 4.0 * iters * 16.0 * 32768.0 / (ms * 1e9);
    return LGA_OK;
}
