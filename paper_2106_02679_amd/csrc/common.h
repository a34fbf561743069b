// Shared device/host declarations for the layer-stack kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lga {

typedef __bf16 bf16;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16;        // IEEE half (section 2.2: the 16-bit format whose gradients need dynamic scaling)
// 4- and 8-element vectors of a 16-bit element type E (bf16 or f16)
template <class E> using x4 = E __attribute__((ext_vector_type(4)));
template <class E> using x8 = E __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// ---- conversions -----------------------------------------------------------------------
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return static_cast<float>(v); }
template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return static_cast<bf16>(v); }
__device__ __forceinline__ float to_f32(f16 v) { return static_cast<float>(v); }
template <> __device__ __forceinline__ f16 from_f32<f16>(float v) { return static_cast<f16>(v); }

// ---- the 16 x 16 x 32 and 32 x 32 x 16 matrix instructions for either 16-bit element type, fp32 accumulate ----
// v_mfma_f32_16x16x32 accumulating in place, acc += a b, with acc held in accumulation registers: written as
// assembly because the builtin leaves the choice of destination to the register allocator, which with all 256
// accumulation registers taken by accumulators gives some products a destination other than their addend and then
// moves accumulators around in the loop.  What the compiler no longer knows about this instruction, the caller
// guarantees: an accumulator is not read by anything but this instruction until at least 32 wait states after its
// last update, and its operands a, b are registers whose loads the compiler still tracks (s_waitcnt).  Two of these
// in a row on one accumulator need one wait state between them (without it the sums come out wrong): the compiler's
// hazard pass puts an s_nop there when they are two asm statements, as here - it does not look inside one.
typedef int i32x4 __attribute__((ext_vector_type(4)));
template <class E> __device__ __forceinline__ void mfma_16x16x32_acc(x8<E> a, x8<E> b, f32x4 &acc);
template <> __device__ __forceinline__ void mfma_16x16x32_acc<bf16>(x8<bf16> a, x8<bf16> b, f32x4 &acc) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(__builtin_bit_cast(i32x4, a)), "v"(__builtin_bit_cast(i32x4, b)));
}
template <> __device__ __forceinline__ void mfma_16x16x32_acc<f16>(x8<f16> a, x8<f16> b, f32x4 &acc) {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(__builtin_bit_cast(i32x4, a)), "v"(__builtin_bit_cast(i32x4, b)));
}
template <class E> __device__ __forceinline__ f32x16 mfma_32x32x16(x8<E> a, x8<E> b, f32x16 c);
template <> __device__ __forceinline__ f32x16 mfma_32x32x16<bf16>(x8<bf16> a, x8<bf16> b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
template <> __device__ __forceinline__ f32x16 mfma_32x32x16<f16>(x8<f16> a, x8<f16> b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// ---- wave / block reductions -------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sum over a block of up to 1024 threads; every thread receives the total.
// `scratch` must hold 16 floats of LDS and may be reused after the call returns.
__device__ __forceinline__ float block_sum(float v, float *scratch) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[w] = v;
    __syncthreads();
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += scratch[i];
    return t;
}

// ---- GELU, tanh form ---------------------------------------------------------------------
// 0.5 u (1 + tanh(c (u + a u^3))), c = sqrt(2/pi), a = 0.044715
constexpr float kGeluC = 0.7978845608028654f;
constexpr float kGeluA = 0.044715f;

// Written with the logistic function: 0.5 (1 + tanh z) = 1 / (1 + exp(-2 z)) =: s, so
//   gelu(u) = u s,   gelu'(u) = s + u s (1 - s) 2 z'(u),   z'(u) = c (1 + 3 a u^2).
// v_exp_f32 and v_rcp_f32 (1 ulp each) instead of the full-precision exp and division; exp overflows to +inf for
// very negative z, whose reciprocal is the correct limit 0.
__device__ __forceinline__ float gelu_logistic(float u, float u2) {
    constexpr float k = -2.0f * kGeluC * 1.4426950408889634f;            // exp(-2 z) = 2^(k u (1 + a u^2))
    const float e = __builtin_amdgcn_exp2f((k * u) * fmaf(kGeluA, u2, 1.0f));
    return __builtin_amdgcn_rcpf(e + 1.0f);
}
__device__ __forceinline__ float gelu_f(float u) { return u * gelu_logistic(u, u * u); }
__device__ __forceinline__ float gelu_grad_f(float u) {
    const float u2 = u * u;
    const float s = gelu_logistic(u, u2);
    const float dz2 = fmaf(6.0f * kGeluA * kGeluC, u2, 2.0f * kGeluC);   // 2 z'(u)
    return fmaf(u * fmaf(-s, s, s), dz2, s);
}

// ---- GEMM epilogues ----------------------------------------------------------------------
// C[m, n] = f(sum_k A(m,k) B(k,n)).  All outputs are row-major with leading dimension ldc.
enum Epilogue : int {
    EPI_STORE = 0,       // out = acc
    EPI_BIAS = 1,        // out = acc + bias[n]
    EPI_BIAS_RESID = 2,  // out = acc + bias[n] + aux[m, n]                 (aux: residual stream)
    EPI_BIAS_GELU = 3,   // out2 = acc + bias[n]; out = gelu(out2)           (out2: pre-activation)
    EPI_MUL_DGELU = 4,   // out = acc * gelu'(aux[m, n])                     (aux: pre-activation)
    EPI_ACCUM_F32 = 5    // outf = beta * outf + acc (fp32 gradient buffer)
};

template <class T> struct GemmParams {
    const T *A;      // see kernels for the storage convention selected by the transpose flags
    const T *B;
    int M, N, K;
    int lda, ldb, ldc;
    T *out;          // main output (activation type)
    T *out2;         // second output (EPI_BIAS_GELU)
    float *outf;     // fp32 output (EPI_ACCUM_F32)
    const float *bias;
    const T *aux;    // leading dimension ldc
    float beta;
    // EPI_ACCUM_F32 with few output tiles: scratch for partial results of slices of the k range (see
    // gemm_splitk_slices); NULL or too small = never split.
    float *partial;
    size_t partial_floats;
    // set by the launcher when it splits: number of k slices, k elements per slice (a multiple of 64)
    int ksplit, kchunk;
    // batch > 1: that many independent products of the same shape in one launch; problem z reads A + z strideA and
    // B + z strideB and writes every output (and reads aux) at + z strideC (elements).  Not combined with a split k range.
    int batch;
    long long strideA, strideB, strideC;
    // Products with a causal mask (M = N = positions, or K = positions): what a tile may leave out because its
    // operand or its consumer is zero there.  0: nothing.  1: tiles entirely above the diagonal (n > every m of the
    // tile) are not computed and not written.  2: the contraction index stops at the tile's last row (k <= m).
    // 3: it starts at the tile's first row (k >= m), rounded down to a whole k tile.
    int tri;
    // set by the launcher for the 256 x 256-tile kernel when the tile grid is a whole number of 16 x 16 blocks: the 256
    // workgroups in flight - 32 per XCD - work on one such block together, each XCD on an 8 x 4 part of it
    int sblock;
};

}  // namespace lga
