// Softmax attention for head sizes that have no fused MFMA kernel (d_h > 160: the X_[x] family of table B.1 has
// d_h = 2 x, 216 for X_108 and 320 for X_160), built from the library's own batched 16-bit GEMMs and two row
// kernels.  The fused kernels keep a query block's operands and accumulators in registers, which ends at d_h = 160;
// here the score matrix of every head goes through memory instead (fp32, so that the softmax sees unrounded scores):
//
//   forward    S = Q K^T                         batched GEMM over the heads, fp32 result
//              P = softmax(S / sqrt(d_h)), lse   row kernel (one wavefront per row), P rounded to 16 bits
//              O = P V                           batched GEMM
//   backward   S = Q K^T ; dP = dO V^T           batched GEMMs, fp32 results
//              P = exp(S / sqrt(d_h) - lse), delta = rowsum(dO * O), dS = P * (dP - delta) / sqrt(d_h)     row kernel
//              dV = P^T dO ; dQ = dS K ; dK = dS^T Q                                                        batched GEMMs
//
// Heads are operands of one launch (GemmParams::batch), sequences are looped over on the host.  With the causal
// mask the row kernels write the masked half of P and dS as zeros and never read the masked half of S and dP, so the
// products leave out what that makes superfluous (GemmParams::tri): score tiles above the diagonal, and the part of
// every contraction over positions that meets only zeros.  The workspace holds
// S, dP (fp32) and P, dS (16 bits) of as many heads as fit: 12 s^2 bytes per head.
#include <algorithm>
#include <type_traits>

#include "kernels.h"

namespace lga {

namespace {

constexpr int kRowsPerBlock = 4;       // one wavefront per row

// P[z][i][j] = softmax_j(scale * S[z][i][j]) over the visible j, lse = log sum_j exp(scale * S[z][i][j]).
// Rows are s floats, 16-byte aligned (s is a multiple of 8).  z counts the heads of this launch.
template <class E>
__global__ __launch_bounds__(64 * kRowsPerBlock) void attn_softmax_rows_kernel(const float *__restrict__ S, E *__restrict__ P,
                                                                               float *__restrict__ lse, int s, int nz,
                                                                               float scale, int causal) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (row >= (long long)nz * s) return;
    const int i = (int)(row % s);
    const int jend = causal ? i + 1 : s;                 // visible keys: [0, jend)
    const float *srow = S + row * s;
    E *prow = P + row * s;
    const float c2 = scale * 1.4426950408889634f;        // work in the log2 domain
    // pass 1: running maximum and sum per lane (4 keys at a time), then across the wavefront
    float m = -INFINITY, l = 0.f;
    for (int j0 = lane * 4; j0 < jend; j0 += 256) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(srow + j0);
        float x[4] = {v[0] * c2, v[1] * c2, v[2] * c2, v[3] * c2};
        float mx = m;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j0 + e < jend) mx = fmaxf(mx, x[e]);
        float add = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (j0 + e < jend) add += __builtin_amdgcn_exp2f(x[e] - mx);
        l = l * __builtin_amdgcn_exp2f(m - mx) + add;      // m = -inf at first: exp2(-inf) = 0, l = 0
        m = mx;
    }
    const float mw = wave_max(m);
    l = (m == -INFINITY) ? 0.f : l * __builtin_amdgcn_exp2f(m - mw);
    const float lw = wave_sum(l);
    const float inv = 1.0f / lw;
    if (lane == 0) lse[row] = (mw + __log2f(lw)) * 0.6931471805599453f;
    // pass 2: write the probabilities, zeros beyond the visible keys
    for (int j0 = lane * 4; j0 < s; j0 += 256) {
        x4<E> o;
        if (j0 < jend) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(srow + j0);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (E)((j0 + e < jend) ? __builtin_amdgcn_exp2f(v[e] * c2 - mw) * inv : 0.f);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (E)0.f;
        }
        *reinterpret_cast<x4<E> *>(prow + j0) = o;
    }
}

// Backward row kernel.  For row (z, i): delta = sum_c dO[i][c] O[i][c]; P[j] = exp(scale S[j] - lse); dS[j] =
// P[j] (dP[j] - delta) scale; both written in 16 bits, zeros beyond the visible keys.
// o_rows / do_rows point at this sequence's first head of the launch: row i of head z is at + i * d + z * dh.
template <class E>
__global__ __launch_bounds__(64 * kRowsPerBlock) void attn_ds_rows_kernel(const float *__restrict__ S, const float *__restrict__ dP,
                                                                          const float *__restrict__ lse, const E *__restrict__ o_rows,
                                                                          const E *__restrict__ do_rows, E *__restrict__ P,
                                                                          E *__restrict__ dS, float *__restrict__ delta, int s,
                                                                          int nz, int dh, int d, float scale, int causal) {
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (row >= (long long)nz * s) return;
    const int i = (int)(row % s), z = (int)(row / s);
    const int jend = causal ? i + 1 : s;
    const E *orow = o_rows + (size_t)i * d + (size_t)z * dh, *dorow = do_rows + (size_t)i * d + (size_t)z * dh;
    float dl = 0.f;
    for (int c = lane * 8; c < dh; c += 512) {           // dh is a multiple of 8
        const x8<E> a = *reinterpret_cast<const x8<E> *>(orow + c), b = *reinterpret_cast<const x8<E> *>(dorow + c);
#pragma unroll
        for (int e = 0; e < 8; ++e) dl += (float)a[e] * (float)b[e];
    }
    dl = wave_sum(dl);
    if (lane == 0) delta[row] = dl;
    const float c2 = scale * 1.4426950408889634f, lse2 = lse[row] * 1.4426950408889634f;
    const float *srow = S + row * s, *dprow = dP + row * s;
    E *prow = P + row * s, *dsrow = dS + row * s;
    for (int j0 = lane * 4; j0 < s; j0 += 256) {
        x4<E> po, dso;
        if (j0 < jend) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(srow + j0), g = *reinterpret_cast<const f32x4 *>(dprow + j0);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float p = (j0 + e < jend) ? __builtin_amdgcn_exp2f(v[e] * c2 - lse2) : 0.f;
                po[e] = (E)p;
                dso[e] = (E)((j0 + e < jend) ? p * (g[e] - dl) * scale : 0.f);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                po[e] = (E)0.f;
                dso[e] = (E)0.f;
            }
        }
        *reinterpret_cast<x4<E> *>(prow + j0) = po;
        *reinterpret_cast<x4<E> *>(dsrow + j0) = dso;
    }
}

// Explicit instantiations: the host compiler does not always emit the launch stub of a kernel template from its use
// in the launchers below alone.
#define LGA_INSTANTIATE_ROW_KERNELS(E)                                                                          \
    template __global__ void attn_softmax_rows_kernel<E>(const float *, E *, float *, int, int, float, int);   \
    template __global__ void attn_ds_rows_kernel<E>(const float *, const float *, const float *, const E *,   \
                                                    const E *, E *, E *, float *, int, int, int, int, float, int)
LGA_INSTANTIATE_ROW_KERNELS(bf16);
LGA_INSTANTIATE_ROW_KERNELS(f16);
#undef LGA_INSTANTIATE_ROW_KERNELS

// Workspace carving for `hc` heads of one sequence.
template <class E> struct Carve {
    float *S, *dP;
    E *P, *dS;
    Carve(void *ws, int hc, int s) {
        const size_t n = (size_t)hc * s * s;
        S = static_cast<float *>(ws);
        dP = S + n;
        P = reinterpret_cast<E *>(dP + n);
        dS = P + n;
    }
};

int heads_per_pass(AttnShape sh, size_t ws_bytes) {
    const size_t per_head = attn_gemm_workspace_bytes(sh.s, 1);
    return (int)std::min<size_t>((size_t)sh.heads, ws_bytes / per_head);
}

template <class E> GemmParams<E> batched(int hc, int M, int N, int K) {
    GemmParams<E> g{};
    g.M = M; g.N = N; g.K = K;
    g.batch = hc;
    return g;
}

}  // namespace

size_t attn_gemm_workspace_bytes(int s, int heads) { return (size_t)heads * s * s * 12; }

bool attn_gemm_supports(AttnShape sh, size_t ws_bytes) {
    return sh.s % 8 == 0 && sh.dh % 8 == 0 && sh.s <= 32768 && ws_bytes >= attn_gemm_workspace_bytes(sh.s, 1);
}

template <class E>
void launch_attn_fwd_gemm(const E *qkv, E *out, float *lse, AttnShape sh, void *ws, size_t ws_bytes, hipStream_t st) {
    if (sh.n_seq == 0 || sh.s == 0) return;
    const int s = sh.s, dh = sh.dh, d = sh.heads * dh, hc_max = heads_per_pass(sh, ws_bytes);
    const float scale = 1.0f / sqrtf((float)dh);
    for (int b = 0; b < sh.n_seq; ++b) {
        const E *seq = qkv + (size_t)b * s * 3 * d;
        for (int h0 = 0; h0 < sh.heads; h0 += hc_max) {
            const int hc = std::min(hc_max, sh.heads - h0);
            Carve<E> w(ws, hc, s);
            // S_h = Q_h K_h^T
            GemmParams<E> g = batched<E>(hc, s, s, dh);
            g.A = seq + (size_t)h0 * dh; g.lda = 3 * d; g.strideA = dh;
            g.B = seq + d + (size_t)h0 * dh; g.ldb = 3 * d; g.strideB = dh;
            g.outf = w.S; g.ldc = s; g.strideC = (long long)s * s;
            g.tri = sh.causal ? 1 : 0;
            launch_gemm_mfma<E>(g, true, true, EPI_ACCUM_F32, st);
            {
                const long long rows = (long long)hc * s;
                ProfScope scope("attn_softmax_rows_kernel", 5.0 * rows * s, 6.0 * rows * s, st);
                hipLaunchKernelGGL(attn_softmax_rows_kernel<E>, dim3((unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock)),
                                   dim3(64 * kRowsPerBlock), 0, st, w.S, w.P, lse + ((size_t)b * sh.heads + h0) * s, s, hc,
                                   scale, sh.causal);
            }
            // O_h = P_h V_h
            g = batched<E>(hc, s, dh, s);
            g.A = w.P; g.lda = s; g.strideA = (long long)s * s;
            g.B = seq + 2 * d + (size_t)h0 * dh; g.ldb = 3 * d; g.strideB = dh;
            g.out = out + (size_t)b * s * d + (size_t)h0 * dh; g.ldc = d; g.strideC = dh;
            g.tri = sh.causal ? 2 : 0;                     // keys up to the query
            launch_gemm_mfma<E>(g, true, false, EPI_STORE, st);
        }
    }
}

template <class E>
void launch_attn_bwd_gemm(const E *qkv, const E *out, const float *lse, const E *dout, E *dqkv, float *delta,
                          AttnShape sh, void *ws, size_t ws_bytes, hipStream_t st) {
    if (sh.n_seq == 0 || sh.s == 0) return;
    const int s = sh.s, dh = sh.dh, d = sh.heads * dh, hc_max = heads_per_pass(sh, ws_bytes);
    const float scale = 1.0f / sqrtf((float)dh);
    const long long ss = (long long)s * s;
    for (int b = 0; b < sh.n_seq; ++b) {
        const E *seq = qkv + (size_t)b * s * 3 * d;
        E *dseq = dqkv + (size_t)b * s * 3 * d;
        for (int h0 = 0; h0 < sh.heads; h0 += hc_max) {
            const int hc = std::min(hc_max, sh.heads - h0);
            Carve<E> w(ws, hc, s);
            const E *q = seq + (size_t)h0 * dh, *k = seq + d + (size_t)h0 * dh, *v = seq + 2 * d + (size_t)h0 * dh;
            const E *o = out + (size_t)b * s * d + (size_t)h0 * dh, *dO = dout + (size_t)b * s * d + (size_t)h0 * dh;
            // S_h = Q_h K_h^T ; dP_h = dO_h V_h^T
            GemmParams<E> g = batched<E>(hc, s, s, dh);
            g.A = q; g.lda = 3 * d; g.strideA = dh;
            g.B = k; g.ldb = 3 * d; g.strideB = dh;
            g.outf = w.S; g.ldc = s; g.strideC = ss;
            g.tri = sh.causal ? 1 : 0;
            launch_gemm_mfma<E>(g, true, true, EPI_ACCUM_F32, st);
            g = batched<E>(hc, s, s, dh);
            g.A = dO; g.lda = d; g.strideA = dh;
            g.B = v; g.ldb = 3 * d; g.strideB = dh;
            g.outf = w.dP; g.ldc = s; g.strideC = ss;
            g.tri = sh.causal ? 1 : 0;
            launch_gemm_mfma<E>(g, true, true, EPI_ACCUM_F32, st);
            {
                const long long rows = (long long)hc * s;
                const size_t stat = ((size_t)b * sh.heads + h0) * s;
                ProfScope scope("attn_ds_rows_kernel", 6.0 * rows * s, 12.0 * rows * s, st);
                hipLaunchKernelGGL(attn_ds_rows_kernel<E>, dim3((unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock)),
                                   dim3(64 * kRowsPerBlock), 0, st, w.S, w.dP, lse + stat, o, dO, w.P, w.dS, delta + stat, s, hc,
                                   dh, d, scale, sh.causal);
            }
            // dV_h = P_h^T dO_h      (contraction over the queries: P is the m-contiguous operand)
            g = batched<E>(hc, s, dh, s);
            g.A = w.P; g.lda = s; g.strideA = ss;
            g.B = dO; g.ldb = d; g.strideB = dh;
            g.out = dseq + 2 * d + (size_t)h0 * dh; g.ldc = 3 * d; g.strideC = dh;
            g.tri = sh.causal ? 3 : 0;                     // queries from the key on
            launch_gemm_mfma<E>(g, false, false, EPI_STORE, st);
            // dQ_h = dS_h K_h
            g = batched<E>(hc, s, dh, s);
            g.A = w.dS; g.lda = s; g.strideA = ss;
            g.B = k; g.ldb = 3 * d; g.strideB = dh;
            g.out = dseq + (size_t)h0 * dh; g.ldc = 3 * d; g.strideC = dh;
            g.tri = sh.causal ? 2 : 0;
            launch_gemm_mfma<E>(g, true, false, EPI_STORE, st);
            // dK_h = dS_h^T Q_h
            g = batched<E>(hc, s, dh, s);
            g.A = w.dS; g.lda = s; g.strideA = ss;
            g.B = q; g.ldb = 3 * d; g.strideB = dh;
            g.out = dseq + d + (size_t)h0 * dh; g.ldc = 3 * d; g.strideC = dh;
            g.tri = sh.causal ? 3 : 0;
            launch_gemm_mfma<E>(g, false, false, EPI_STORE, st);
        }
    }
}

#define LGA_INSTANTIATE_ATTN_GEMM(E)                                                                               \
    template void launch_attn_fwd_gemm<E>(const E *, E *, float *, AttnShape, void *, size_t, hipStream_t);       \
    template void launch_attn_bwd_gemm<E>(const E *, const E *, const float *, const E *, E *, float *, AttnShape, \
                                          void *, size_t, hipStream_t)
LGA_INSTANTIATE_ATTN_GEMM(bf16);
LGA_INSTANTIATE_ATTN_GEMM(f16);
#undef LGA_INSTANTIATE_ATTN_GEMM

}  // namespace lga
