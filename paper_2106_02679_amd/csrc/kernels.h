// Host-side launchers of every HIP kernel of the layer-stack library.
// Each launcher checks nothing: shapes are validated by the callers (stack.hip, ops_api.hip).
#pragma once

#include "common.h"
#include "prof.h"

namespace lga {

// ---- one-time set-up ----------------------------------------------------------------------
// Kernels that use more dynamic LDS than a launch may ask for by default (the attention kernels, the large-tile
// GEMM) have their limit raised here, once per process, before anything is launched: lga_init_stack calls it, and
// so does every launcher of such a kernel (a flag test after the first call), so the op-level entry points need no
// stack.  It must not run for the first time on a stream that is being captured into a graph - which is why the
// stack-level entry points call it at init and refuse capturing streams.
hipError_t prepare_kernels();
hipError_t attn_prepare_kernels();      // attention_bf16.hip's part
hipError_t gemm_prepare_kernels();      // gemm_bf16.hip's part

// ---- element-wise / row kernels (rowops.hip) ---------------------------------------------
// fp32 -> 16-bit copy of a parameter vector ("restore": parameters converted to 16 bits before use); E = bf16 or f16.
template <class E> void launch_cast_f32_to_16(const float *src, E *dst, size_t n, hipStream_t s);
// Counter-based N(0, std^2) fill: element i gets a value that depends only on (seed, i).
void launch_fill_normal(float *dst, size_t n, float std, uint64_t seed, hipStream_t s);
void launch_fill_const(float *dst, size_t n, float value, hipStream_t s);

// LayerNorm forward over rows of length d.  Writes y = xhat * g + b and the row statistics.
template <class T>
void launch_layernorm_fwd(const T *x, const float *g, const float *b, T *y, float *mean, float *rstd,
                          int rows, int d, float eps, hipStream_t s);
// LayerNorm backward w.r.t. the input, fused with the residual add:
//   dx = resid + rstd * (g dy - mean_row(g dy) - xhat * mean_row(g dy xhat))
// dbeta != NULL: also the gradients of the LayerNorm bias and gain,
//   dbeta[c] = beta * dbeta[c] + sum_r dy[r, c],   dgamma[c] = beta * dgamma[c] + sum_r dy[r, c] xhat[r, c],
// added up inside the same kernel where the width allows, by the column-sum kernels otherwise; partial then holds
// layernorm_bwd_partial_floats(rows, d) floats.
size_t layernorm_bwd_partial_floats(int rows, int d);
template <class T>
void launch_layernorm_bwd_dx(const T *dy, const T *x, const float *mean, const float *rstd, const float *g,
                             const T *resid, T *dx, int rows, int d, hipStream_t s, float beta = 0.f,
                             float *dbeta = nullptr, float *dgamma = nullptr, float *partial = nullptr);

// Column sums over rows, in two deterministic passes through `partial`:
//   out0[c] = beta * out0[c] + sum_r a[r, c]
//   out1[c] = beta * out1[c] + sum_r a[r, c] * (x[r, c] - mean[r]) * rstd[r]     (only if out1 != NULL)
// a and x have leading dimension ld.  partial must hold colsum_partial_floats(rows, cols) floats.
// timed = false keeps the launch out of the per-launch profile (no events are created for it).
size_t colsum_partial_floats(int rows, int cols);
template <class T>
void launch_colsum(const T *a, const T *x, const float *mean, const float *rstd, int rows, int cols, int ld,
                   float beta, float *out0, float *out1, float *partial, hipStream_t s, bool timed = true);

// out[c][r] = in[r][c] for matrices of 16-bit elements of any format; R, C, ldi, ldo multiples of 8, 16-byte
// aligned bases.
void launch_transpose16(const void *in, void *out, int R, int C, long ldi, long ldo, hipStream_t s);
// The same for format E, and out0[c] = beta * out0[c] + sum_r in[r, c] from the tiles as they pass through the
// transposing kernel (partial: colsum_partial_floats(R, C) floats).
template <class E>
void launch_transpose16_colsum(const E *in, E *out, int R, int C, long ldi, long ldo, float beta, float *out0,
                               float *partial, hipStream_t s);

// 1 into *flag if any of the n values is infinite or not a number (*flag is not cleared here).
void launch_nonfinite_flag(const float *g, size_t n, int *flag, hipStream_t s);

// Adam update of n parameters in place; optionally (w16 != NULL) also writes the 16-bit copy of the new weights in
// format E (bf16 or f16).  The gradient is multiplied by grad_mul before use (1 / loss scale).  skip != NULL: the
// whole update is left out when *skip != 0 (gradient found non-finite).
template <class E>
void launch_adam(float *w, float *m, float *v, const float *g, E *w16, size_t n, float lr, float beta1, float beta2,
                 float eps, int step, float grad_mul, const int *skip, hipStream_t s);

// ---- GEMMs -------------------------------------------------------------------------------
// C[M,N] = sum_k A(m,k) B(k,n), then the epilogue.
//   a_kmajor: A is stored [M][lda] (k contiguous); otherwise [K][lda] (m contiguous).
//   b_kmajor: B is stored [N][ldb] (k contiguous); otherwise [K][ldb] (n contiguous).
// fp32 correctness-mode kernel (plain FMA, LDS tiles):
void launch_gemm_f32(const GemmParams<float> &p, bool a_kmajor, bool b_kmajor, Epilogue epi, hipStream_t s);
// 16-bit MFMA kernel (E = bf16 or f16), fp32 accumulate.  Needs lda, ldb, ldc, N multiples of 8 and 16-byte aligned
// bases.
// Returns false, launching nothing, for a layout / epilogue pair that is not built (gemm_mfma_supports) or a leading
// dimension beyond kGemmMaxLd.
constexpr int kGemmMaxLd = ((1 << 30) - 256) / (2 * 256);      // 2 097 151 elements: row 255 of a tile stays inside the loads' 1 GiB window
bool gemm_mfma_supports(bool a_kmajor, bool b_kmajor, Epilogue epi);
template <class E>
bool launch_gemm_mfma(const GemmParams<E> &p, bool a_kmajor, bool b_kmajor, Epilogue epi, hipStream_t s);
// Into how many slices of the k range launch_gemm_mfma cuts an fp32-accumulating, k-contiguous GEMM whose output has
// too few 256 x 256 tiles to occupy the chip (1 = not at all); it then needs slices * M * N floats of scratch.
// k = 0 asks for the largest count any k would give (for sizing the scratch).
int gemm_splitk_slices(int M, int N, int K);

// ---- causal attention --------------------------------------------------------------------
// qkv: [tokens, 3 d] with columns [Q | K | V], head h at columns h*dh inside each third; tokens =
// n_seq * s, each sequence attends only to itself.  out: [tokens, d].  lse: [n_seq, heads, s] holds
// log(sum_j exp(score_ij)) of the scaled scores.  d = heads * dh.
// causal != 0: position i attends to j <= i (decoder); 0: to its whole sequence (encoder).
struct AttnShape {
    int n_seq, s, heads, dh, causal;
};
template <class T> void launch_attn_fwd_simple(const T *qkv, T *out, float *lse, AttnShape sh, hipStream_t s);
// dqkv: [tokens, 3 d]; delta: scratch [n_seq, heads, s] (row sums of dout * out).
template <class T>
void launch_attn_bwd_simple(const T *qkv, const T *out, const float *lse, const T *dout, T *dqkv, float *delta,
                            AttnShape sh, hipStream_t s);
// MFMA kernels with LDS-resident online softmax (E = bf16 or f16).  Head sizes other than those
// attn_bf16_supports() accepts are routed to the one-wavefront kernels above.
bool attn_bf16_supports(int dh);
template <class E> void launch_attn_fwd_mfma(const E *qkv, E *out, float *lse, AttnShape sh, hipStream_t s);
template <class E>
void launch_attn_bwd_mfma(const E *qkv, const E *out, const float *lse, const E *dout, E *dqkv, float *delta,
                          AttnShape sh, hipStream_t s);

// The same attention for head sizes without a fused kernel, built from batched GEMMs and two row kernels
// (attention_gemm.hip).  Needs s and dh to be multiples of 8 and a workspace of at least
// attn_gemm_workspace_bytes(s, 1) bytes (256-byte aligned); more workspace, up to attn_gemm_workspace_bytes(s, heads),
// lets more heads share a launch.
size_t attn_gemm_workspace_bytes(int s, int heads);
bool attn_gemm_supports(AttnShape sh, size_t ws_bytes);
template <class E>
void launch_attn_fwd_gemm(const E *qkv, E *out, float *lse, AttnShape sh, void *ws, size_t ws_bytes, hipStream_t s);
template <class E>
void launch_attn_bwd_gemm(const E *qkv, const E *out, const float *lse, const E *dout, E *dqkv, float *delta,
                          AttnShape sh, void *ws, size_t ws_bytes, hipStream_t s);

}  // namespace lga
