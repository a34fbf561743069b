// fp32 GEMM for the correctness mode: plain FMA, 64x64x16 LDS tiles, any shape.
// Speed is not a goal here; the bf16 MFMA kernel carries the benchmark.
#include "kernels.h"

namespace lga {

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmParams<float> p, long sam, long sak, long sbk, long sbn) {
    __shared__ float As[TK][TM + 1];
    __shared__ float Bs[TK][TN + 1];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
    const int tr = (tid / 16) * 4, tc = (tid % 16) * 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < p.K; k0 += TK) {
        for (int i = tid; i < TM * TK; i += 256) {
            // map so that consecutive threads walk the contiguous storage direction
            int mm, kk;
            if (sak == 1) { kk = i % TK; mm = i / TK; } else { mm = i % TM; kk = i / TM; }
            const int gm = m0 + mm, gk = k0 + kk;
            As[kk][mm] = (gm < p.M && gk < p.K) ? p.A[gm * sam + gk * sak] : 0.f;
        }
        for (int i = tid; i < TN * TK; i += 256) {
            int nn, kk;
            if (sbk == 1) { kk = i % TK; nn = i / TK; } else { nn = i % TN; kk = i / TN; }
            const int gn = n0 + nn, gk = k0 + kk;
            Bs[kk][nn] = (gn < p.N && gk < p.K) ? p.B[gk * sbk + gn * sbn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < TK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][tr + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tc + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + tr + i;
        if (m >= p.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tc + j;
            if (n >= p.N) continue;
            const size_t idx = (size_t)m * p.ldc + n;
            const float a = acc[i][j];
            if constexpr (EPI == EPI_STORE) {
                p.out[idx] = a;
            } else if constexpr (EPI == EPI_BIAS) {
                p.out[idx] = a + p.bias[n];
            } else if constexpr (EPI == EPI_BIAS_RESID) {
                p.out[idx] = a + p.bias[n] + p.aux[idx];
            } else if constexpr (EPI == EPI_BIAS_GELU) {
                const float u = a + p.bias[n];
                p.out2[idx] = u;
                p.out[idx] = gelu_f(u);
            } else if constexpr (EPI == EPI_MUL_DGELU) {
                p.out[idx] = a * gelu_grad_f(p.aux[idx]);
            } else {
                p.outf[idx] = (p.beta == 0.f ? 0.f : p.beta * p.outf[idx]) + a;
            }
        }
    }
}

}  // namespace

void launch_gemm_f32(const GemmParams<float> &p, bool a_kmajor, bool b_kmajor, Epilogue epi, hipStream_t s) {
    if (p.M == 0 || p.N == 0) return;
    const long sam = a_kmajor ? p.lda : 1, sak = a_kmajor ? 1 : p.lda;
    const long sbn = b_kmajor ? p.ldb : 1, sbk = b_kmajor ? 1 : p.ldb;
    dim3 grid((p.N + TN - 1) / TN, (p.M + TM - 1) / TM), block(256);
    const double mn = (double)p.M * p.N;
    ProfScope scope("gemm_f32_kernel", 2.0 * mn * p.K, 4.0 * ((double)p.M * p.K + (double)p.K * p.N + mn), s);
    switch (epi) {
        case EPI_STORE: hipLaunchKernelGGL(gemm_f32_kernel<EPI_STORE>, grid, block, 0, s, p, sam, sak, sbk, sbn); break;
        case EPI_BIAS: hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS>, grid, block, 0, s, p, sam, sak, sbk, sbn); break;
        case EPI_BIAS_RESID:
            hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS_RESID>, grid, block, 0, s, p, sam, sak, sbk, sbn); break;
        case EPI_BIAS_GELU:
            hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS_GELU>, grid, block, 0, s, p, sam, sak, sbk, sbn); break;
        case EPI_MUL_DGELU:
            hipLaunchKernelGGL(gemm_f32_kernel<EPI_MUL_DGELU>, grid, block, 0, s, p, sam, sak, sbk, sbn); break;
        case EPI_ACCUM_F32:
            hipLaunchKernelGGL(gemm_f32_kernel<EPI_ACCUM_F32>, grid, block, 0, s, p, sam, sak, sbk, sbn); break;
    }
}

}  // namespace lga
