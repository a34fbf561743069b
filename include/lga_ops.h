/*
 * lga_ops.h - kernel-level entry points of the layer-stack library.
 *
 * Each call runs ONE of the kernels that lga_forward_layered / lga_backward_layered are built
 * from, on caller-owned device buffers, so that every kernel can be checked on its own against the
 * CPU oracle at small, ragged shapes.  Same conventions as lga.h: int status codes, validation on
 * the host before any launch, `stream` is a borrowed hipStream_t (NULL = default), calls enqueue
 * and return.  dtype is enum lga_dtype and selects the storage type of activation tensors
 * (float, bfloat16 or IEEE half); statistics, biases, gains and gradients of parameters are always float.
 * "16-bit" below means LGA_BF16 or LGA_FP16: the same kernels on either format.
 */
#ifndef LGA_OPS_H
#define LGA_OPS_H

#include "lga.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Epilogues of lga_op_gemm.  All outputs are row-major [M, N] with leading dimension ldc. */
enum lga_epilogue {
    LGA_EPI_STORE = 0,      /* out = acc */
    LGA_EPI_BIAS = 1,       /* out = acc + bias[n]                          (linear maps, section 5) */
    LGA_EPI_BIAS_RESID = 2, /* out = acc + bias[n] + aux[m,n]               (residual add) */
    LGA_EPI_BIAS_GELU = 3,  /* out2 = acc + bias[n]; out = gelu_tanh(out2)  (feed-forward non-linearity) */
    LGA_EPI_MUL_DGELU = 4,  /* out = acc * gelu_tanh'(aux[m,n]) */
    LGA_EPI_ACCUM_F32 = 5   /* outf = beta * outf + acc, fp32               (weight-gradient accumulation
                               across micro-batches, section 2.5 / section 3) */
};

/* C[M,N] = sum_k A(m,k) B(k,n) followed by an epilogue (appendix C.1: the dense-layer products are
 * the bulk of the computation).
 *  a_kmajor != 0: A is stored [M][lda], k contiguous; else [K][lda], m contiguous.
 *  b_kmajor != 0: B is stored [N][ldb], k contiguous; else [K][ldb], n contiguous.
 * LGA_FP32: any shape.  16-bit (MFMA kernel): lda, ldb, ldc, N - and M when A is m-contiguous, K
 * when either operand is k-contiguous - must be multiples of 8, all pointers 16-byte aligned, and the layout/epilogue
 * pair must be one that is built: (k,k-major) with any epilogue - the layout the layer stack itself
 * uses for all three GEMM families -, (k,n-major) with STORE/BIAS/BIAS_RESID/BIAS_GELU, (m,n-major) with
 * STORE/ACCUM_F32.  Otherwise LGA_ERR_SHAPE. */
int lga_op_gemm(int32_t dtype, int32_t a_kmajor, int32_t b_kmajor, int32_t epilogue, int32_t M, int32_t N, int32_t K,
                const void *A, int32_t lda, const void *B, int32_t ldb, void *out, void *out2, float *outf,
                int32_t ldc, const float *bias, const void *aux, float beta, void *stream);

/* The weight-gradient GEMM as the layer stack runs it (section 3: one accumulation per layer over all micro-batches'
 * tokens): outf[M,N] = beta * outf + sum_k A[m][k] B[n][k], 16-bit operands (dtype) with k contiguous ([M][lda], [N][ldb]), fp32
 * result.  When the output has too few 256 x 256 tiles to occupy the chip (narrow layers) and `scratch` (device, at
 * least lga_op_gemm_splitk_slices(M, N, K) * M * N floats, 16-byte aligned) is given, the k range is cut into that many
 * slices that run as separate workgroups and are then summed in slice order (deterministic); otherwise, or with
 * scratch == NULL, it is lga_op_gemm with LGA_EPI_ACCUM_F32.  Alignment rules as for lga_op_gemm. */
int lga_op_gemm_splitk(int32_t dtype, int32_t M, int32_t N, int32_t K, const void *A, int32_t lda, const void *B,
                       int32_t ldb, float *outf, int32_t ldc, float beta, float *scratch, uint64_t scratch_floats, void *stream);
/* Number of k slices lga_op_gemm_splitk would use (1 = no split); K = 0: the most any K would give. */
int32_t lga_op_gemm_splitk_slices(int32_t M, int32_t N, int32_t K);

/* LayerNorm over rows of length d (biased variance, eps inside the root): y = (x-mean)*rstd*g + b.
 * mean, rstd: [rows] float, written. */
int lga_op_layernorm_fwd(int32_t dtype, const void *x, const float *g, const float *b, void *y, float *mean,
                         float *rstd, int32_t rows, int32_t d, float eps, void *stream);

/* LayerNorm backward fused with the residual add:
 *   dx = resid + rstd * (g*dy - mean_row(g*dy) - xhat * mean_row(g*dy*xhat))
 *   dgamma = beta*dgamma + sum_rows dy*xhat ;  dbeta = beta*dbeta + sum_rows dy
 * The two sums are taken inside the dx kernel from the operands it holds anyway (rows of up to 8192 16-bit or 4096
 * fp32 values; wider rows: by the column-sum kernels, in a pass of their own), block by block into `scratch`, and
 * added up in block order, so the result does not depend on scheduling.
 * scratch: lga_op_layernorm_bwd_scratch_floats(rows, d) floats of device memory, 16-byte aligned. */
int lga_op_layernorm_bwd(int32_t dtype, const void *dy, const void *x, const float *mean, const float *rstd,
                         const float *g, const void *resid, void *dx, float *dgamma, float *dbeta, float beta,
                         float *scratch, int32_t rows, int32_t d, void *stream);
uint64_t lga_op_layernorm_bwd_scratch_floats(int32_t rows, int32_t d);

/* out[c][r] = in[r][c] for matrices of 16-bit elements of either format (in: [R][ldi], out: [C][ldo]); R, C, ldi, ldo multiples of 8,
 * 16-byte aligned.  The stack keeps a transposed 16-bit copy of each weight matrix and transposes the
 * two operands of every weight-gradient GEMM so that all GEMM operands are k-contiguous. */
int lga_op_transpose(const void *in, void *out, int32_t R, int32_t C, int64_t ldi, int64_t ldo, void *stream);

/* lga_op_transpose of a matrix of format `dtype` (LGA_BF16 or LGA_FP16) that also returns its column sums,
 *   sums[c] = beta*sums[c] + sum_r in[r,c],
 * added up tile by tile as the matrix passes through the transposing kernel: the output gradient of a linear map is
 * transposed for the weight-gradient GEMM, and its column sums are the bias gradient (section 3: gradients accumulated
 * per layer), so that gradient costs no pass over memory of its own.  Deterministic (two passes, fixed order).
 * scratch: lga_op_colsum_scratch_floats(R, C) floats of device memory. */
int lga_op_transpose_colsum(int32_t dtype, const void *in, void *out, int32_t R, int32_t C, int64_t ldi, int64_t ldo,
                            float beta, float *sums, float *scratch, void *stream);

/* out[c] = beta*out[c] + sum_r a[r,c]  (bias gradients).  a: [rows][ld]. */
int lga_op_colsum(int32_t dtype, const void *a, int32_t rows, int32_t cols, int32_t ld, float beta, float *out,
                  float *scratch, void *stream);
uint64_t lga_op_colsum_scratch_floats(int32_t rows, int32_t cols);

/* lga_op_colsum for callers that cannot allocate device memory or hand over a workspace: code running under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result as lga_op_colsum (same two
 * kernels, bit-identical output) without `scratch`: the partial sums go to a 16 MiB array that is part of the library's
 * device image (one copy per GPU, kept until the process ends).  The call allocates nothing - no device or host
 * memory, no events (its launches are left out of lga_profile_begin/end) - and enqueues two kernels on `stream`.
 * LGA_ERR_SHAPE if lga_op_colsum_scratch_floats(rows, cols) exceeds lga_op_colsum_static_max_floats() (4 194 304),
 * i.e. if ceil(rows / 128) x 2 x cols floats of partial sums do not fit.
 * All calls on one GPU share that one array: two calls whose kernels may overlap in time (different streams, or
 * different host threads) race on it; calls on one stream are ordered and safe.  Nothing has to be cleared between
 * calls: every partial sum the second kernel reads is written by the first kernel of the same call. */
int lga_op_colsum_static(int32_t dtype, const void *a, int32_t rows, int32_t cols, int32_t ld, float beta, float *out,
                         void *stream);
uint64_t lga_op_colsum_static_max_floats(void);

/* Softmax attention per (sequence, head), scores scaled by 1/sqrt(d_h) (section 5, "Model").
 * causal != 0: position i attends to positions j <= i (decoder); causal == 0: to the whole sequence (encoder).
 *  qkv  [n_seq*s, 3*heads*dh]: columns [Q | K | V], head h at columns h*dh inside each third
 *  out  [n_seq*s, heads*dh]
 *  lse  [n_seq, heads, s] float: log sum_j exp(scaled score_ij)
 * kind 0: one-wavefront-per-position kernel (any dtype, any dh); kind 1: MFMA kernel with
 * LDS-resident online softmax (16-bit, dh a multiple of 8 up to 160; head sizes other than 32, 64, 96, 128, 160
 * run in the next larger of those kernels with the extra columns read as zeros). */
int lga_op_attention_fwd(int32_t dtype, int32_t kind, const void *qkv, void *out, float *lse, int32_t n_seq,
                         int32_t s, int32_t heads, int32_t dh, int32_t causal, void *stream);
/* dqkv [n_seq*s, 3*heads*dh] written; delta [n_seq, heads, s] float scratch (written). */
int lga_op_attention_bwd(int32_t dtype, int32_t kind, const void *qkv, const void *out, const float *lse,
                         const void *dout, void *dqkv, float *delta, int32_t n_seq, int32_t s, int32_t heads,
                         int32_t dh, int32_t causal, void *stream);

/* The same attention for head sizes beyond the fused kernels (table B.1's X_[x] family has d_h = 2 x: 216, 320), built
 * from batched GEMMs over the heads with the score matrices in a workspace: S = Q K^T in fp32, a row kernel for the
 * softmax (P rounded to 16 bits) and O = P V; backward S and dP = dO V^T in fp32, a row kernel for P, delta and dS, then
 * dV = P^T dO, dQ = dS K, dK = dS^T Q.  Arguments and results as above (16-bit dtypes only).  s and dh multiples of 8,
 * s <= 32768.  workspace: device, 256-byte aligned, at least lga_op_attention_gemm_workspace_bytes(s, 1) = 12 s^2 bytes;
 * up to ..._bytes(s, heads) lets that many heads share each launch.  Contents are scratch. */
uint64_t lga_op_attention_gemm_workspace_bytes(int32_t s, int32_t heads);
int lga_op_attention_gemm_fwd(int32_t dtype, const void *qkv, void *out, float *lse, int32_t n_seq, int32_t s,
                              int32_t heads, int32_t dh, int32_t causal, void *workspace, uint64_t workspace_bytes,
                              void *stream);
int lga_op_attention_gemm_bwd(int32_t dtype, const void *qkv, const void *out, const float *lse, const void *dout,
                              void *dqkv, float *delta, int32_t n_seq, int32_t s, int32_t heads, int32_t dh,
                              int32_t causal, void *workspace, uint64_t workspace_bytes, void *stream);

/* One Adam update of n parameters in place (w, m, v fp32; g fp32 read-only); if w16 != NULL the new
 * weights are also written in the 16-bit format w16_dtype (section 2.5: 16-bit copy for the next use).
 * adam->loss_scale divides the gradient first; with adam->skip_nonfinite, *nonfinite (device int32, required then)
 * is set to whether g holds an infinity or NaN, and if it does nothing else is written (see lga_adam). */
int lga_op_adam(float *w, float *m, float *v, const float *g, void *w16, int32_t w16_dtype, uint64_t n,
                const lga_adam *adam, int32_t *nonfinite, void *stream);

/* Calibration for the benchmark tools: the bf16 MFMA rate (TFLOP/s, executed) that the GPU sustains on register
 * operands alone - one workgroup of four wavefronts per CU, each issuing iters x 32 v_mfma_f32_16x16x32_bf16 (the GEMM
 * kernel's instruction, in that kernel's order: two products in a row on each of 16 accumulators), no memory traffic.  mode 0: operand values in [0.5, 1) with random mantissas and signs (what the power
 * management allows on realistic data); 1: all operand values 1.0 (approaches the nominal peak).
 * sink: device, >= 65536 floats, overwritten.  iters in 1 .. 2^23.  Synchronous: returns after the kernel has run.
 * tflops: host. */
int lga_op_mfma_rate(int32_t iters, int32_t mode, float *sink, double *tflops, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LGA_OPS_H */
