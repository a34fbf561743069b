// Kernel-level C ABI (include/lga_ops.h): one kernel per call on caller-owned device buffers.
#include "../../include/lga_ops.h"

#include <mutex>
#include <string>

#include "kernels.h"

using namespace lga;

namespace lga {
bool attn_bf16_supports(int dh);
int set_last_error(int code, const char *msg);
}  // namespace lga

namespace {

int err(int code, const char *msg) { return lga::set_last_error(code, msg); }

bool a16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int done(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return err(LGA_ERR_HIP, (std::string(what) + ": " + hipGetErrorString(e)).c_str());
    return LGA_OK;
}

bool dtype_ok(int32_t dt) { return dt == LGA_FP32 || dt == LGA_BF16 || dt == LGA_FP16; }
bool dtype16(int32_t dt) { return dt == LGA_BF16 || dt == LGA_FP16; }

// body(E{}) with E = the 16-bit element type that dt names
template <class F> void with16(int32_t dt, F &&body) {
    if (dt == LGA_FP16) body(f16{});
    else body(bf16{});
}
template <class E> const E *in16(const void *p) { return static_cast<const E *>(p); }
template <class E> E *out16(void *p) { return static_cast<E *>(p); }

// ---- lga_op_colsum_static: the column sums with their partial results in memory that is part of the library's image
// One copy of this array exists on every GPU the library's code object is loaded on, at its own address there, for as
// long as the process lives.  In host code its name is only a handle for hipGetSymbolAddress; the address the kernels
// get is looked up once per device and kept.
constexpr size_t kStaticScratchFloats = (size_t)4 << 20;         // 16 MiB
static __device__ __align__(256) float static_scratch[kStaticScratchFloats];

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
float *g_static_ptr[kMaxDevices];                                // per device, null until first used there

// Address of the current device's copy of static_scratch (looked up on the first call on that device).
int static_scratch_ptr(float **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return err(LGA_ERR_HIP, (std::string("hipGetDevice: ") + hipGetErrorString(e)).c_str());
    if (dev < 0 || dev >= kMaxDevices) return err(LGA_ERR_HIP, "device index out of the supported range");
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return err(LGA_ERR_HIP, (std::string("hipGetSymbolAddress(static_scratch): ") + hipGetErrorString(e)).c_str());
        }
        g_static_ptr[dev] = static_cast<float *>(p);
    }
    *out = g_static_ptr[dev];
    return LGA_OK;
}

}  // namespace

extern "C" {

uint64_t lga_op_colsum_static_max_floats(void) { return kStaticScratchFloats; }

int lga_op_colsum_static(int32_t dtype, const void *a, int32_t rows, int32_t cols, int32_t ld, float beta, float *out,
                         void *stream) {
    if (!dtype_ok(dtype)) return err(LGA_ERR_ARG, "bad dtype");
    if (rows < 0 || cols < 0 || ld < cols) return err(LGA_ERR_SHAPE, "bad shape");
    if ((!a && rows > 0) || !out) return err(LGA_ERR_ARG, "NULL argument");
    const size_t need = colsum_partial_floats(rows, cols);
    if (need > kStaticScratchFloats)
        return err(LGA_ERR_SHAPE, ("lga_op_colsum_static: rows x cols needs " + std::to_string(need) +
                                   " floats of partial sums, the built-in scratch holds " +
                                   std::to_string(kStaticScratchFloats) + " (use lga_op_colsum with a workspace)").c_str());
    float *scratch = nullptr;
    if (int rc = static_scratch_ptr(&scratch)) return rc;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // Every partial sum the second pass reads is written by the first pass of the same call, so nothing needs to be
    // cleared between calls.  timed = false: no events are created for these launches.
    if (dtype == LGA_FP32)
        launch_colsum<float>(static_cast<const float *>(a), nullptr, nullptr, nullptr, rows, cols, ld, beta, out, nullptr,
                             scratch, s, false);
    else
        with16(dtype, [&](auto tag) {
            using E = decltype(tag);
            launch_colsum<E>(in16<E>(a), nullptr, nullptr, nullptr, rows, cols, ld, beta, out, nullptr, scratch, s, false);
        });
    return done("lga_op_colsum_static");
}

int lga_op_gemm(int32_t dtype, int32_t a_kmajor, int32_t b_kmajor, int32_t epilogue, int32_t M, int32_t N, int32_t K,
                const void *A, int32_t lda, const void *B, int32_t ldb, void *out, void *out2, float *outf,
                int32_t ldc, const float *bias, const void *aux, float beta, void *stream) {
    if (!dtype_ok(dtype)) return err(LGA_ERR_ARG, "bad dtype");
    if (epilogue < LGA_EPI_STORE || epilogue > LGA_EPI_ACCUM_F32) return err(LGA_ERR_ARG, "bad epilogue");
    if (M < 0 || N < 0 || K < 0) return err(LGA_ERR_SHAPE, "negative size");
    if ((M > 0 && N > 0) && (!A || !B) && K > 0) return err(LGA_ERR_ARG, "A or B is NULL");
    const bool akm = a_kmajor != 0, bkm = b_kmajor != 0;
    if (lda < (akm ? K : M) || ldb < (bkm ? K : N) || ldc < N) return err(LGA_ERR_SHAPE, "leading dimension too small");
    const Epilogue e = static_cast<Epilogue>(epilogue);
    if (e == EPI_ACCUM_F32 ? !outf : !out) return err(LGA_ERR_ARG, "output pointer is NULL");
    if ((e == EPI_BIAS || e == EPI_BIAS_RESID || e == EPI_BIAS_GELU) && !bias) return err(LGA_ERR_ARG, "bias is NULL");
    if ((e == EPI_BIAS_RESID || e == EPI_MUL_DGELU) && !aux) return err(LGA_ERR_ARG, "aux is NULL");
    if (e == EPI_BIAS_GELU && !out2) return err(LGA_ERR_ARG, "out2 is NULL");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dtype == LGA_FP32) {
        GemmParams<float> p{};
        p.A = static_cast<const float *>(A); p.B = static_cast<const float *>(B);
        p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
        p.out = static_cast<float *>(out); p.out2 = static_cast<float *>(out2); p.outf = outf;
        p.bias = bias; p.aux = static_cast<const float *>(aux); p.beta = beta;
        launch_gemm_f32(p, akm, bkm, e, s);
    } else {
        if (lda % 8 || ldb % 8 || ldc % 8 || N % 8 || ((akm || bkm) && K % 8) || (!akm && M % 8))
            return err(LGA_ERR_SHAPE, "16-bit GEMM needs lda, ldb, ldc, N (K if an operand is k-contiguous, M if A is "
                                      "m-contiguous) to be multiples of 8");
        if (!a16(A) || !a16(B) || !a16(out) || !a16(out2) || !a16(outf) || !a16(bias) || !a16(aux))
            return err(LGA_ERR_SHAPE, "16-bit GEMM needs 16-byte aligned pointers");
        bool ok = false;
        if (akm && !bkm) ok = e == EPI_STORE || e == EPI_BIAS || e == EPI_BIAS_RESID || e == EPI_BIAS_GELU;
        else if (akm && bkm) ok = true;
        else if (!akm && !bkm) ok = e == EPI_STORE || e == EPI_ACCUM_F32;
        if (!ok || !gemm_mfma_supports(akm, bkm, e)) return err(LGA_ERR_SHAPE, "16-bit GEMM: this layout/epilogue pair is not built");
        if (lda > kGemmMaxLd || ldb > kGemmMaxLd)
            return err(LGA_ERR_SHAPE, "16-bit GEMM: lda and ldb must not exceed 2 097 151 elements (the kernels address a "
                                      "tile's 256 rows with 32-bit byte offsets inside a 1 GiB window)");
        bool launched = true;
        with16(dtype, [&](auto tag) {
            using E = decltype(tag);
            GemmParams<E> p{};
            p.A = in16<E>(A); p.B = in16<E>(B);
            p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
            p.out = out16<E>(out); p.out2 = out16<E>(out2); p.outf = outf;
            p.bias = bias; p.aux = in16<E>(aux); p.beta = beta;
            launched = launch_gemm_mfma<E>(p, akm, bkm, e, s);
        });
        if (!launched) return err(LGA_ERR_SHAPE, "16-bit GEMM: the launcher refused these arguments");
    }
    return done("lga_op_gemm");
}

int32_t lga_op_gemm_splitk_slices(int32_t M, int32_t N, int32_t K) {
    if (M < 1 || N < 1 || K < 0) return 1;
    return gemm_splitk_slices(M, N, K);
}

int lga_op_gemm_splitk(int32_t dtype, int32_t M, int32_t N, int32_t K, const void *A, int32_t lda, const void *B, int32_t ldb,
                       float *outf, int32_t ldc, float beta, float *scratch, uint64_t scratch_floats, void *stream) {
    if (!dtype16(dtype)) return err(LGA_ERR_ARG, "dtype must be LGA_BF16 or LGA_FP16");
    if (M < 0 || N < 0 || K < 0) return err(LGA_ERR_SHAPE, "negative size");
    if (!A || !B || !outf) return err(LGA_ERR_ARG, "NULL argument");
    if (lda < K || ldb < K || ldc < N) return err(LGA_ERR_SHAPE, "leading dimension too small");
    if (lda % 8 || ldb % 8 || ldc % 8 || N % 8 || K % 8)
        return err(LGA_ERR_SHAPE, "16-bit GEMM needs lda, ldb, ldc, N and K to be multiples of 8");
    if (!a16(A) || !a16(B) || !a16(outf) || !a16(scratch)) return err(LGA_ERR_SHAPE, "16-bit GEMM needs 16-byte aligned pointers");
    if (lda > kGemmMaxLd || ldb > kGemmMaxLd)
        return err(LGA_ERR_SHAPE, "16-bit GEMM: lda and ldb must not exceed 2 097 151 elements");
    bool launched = true;
    with16(dtype, [&](auto tag) {
        using E = decltype(tag);
        GemmParams<E> p{};
        p.A = in16<E>(A); p.B = in16<E>(B);
        p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc;
        p.outf = outf; p.beta = beta;
        p.partial = scratch; p.partial_floats = scratch ? scratch_floats : 0;
        launched = launch_gemm_mfma<E>(p, true, true, EPI_ACCUM_F32, reinterpret_cast<hipStream_t>(stream));
    });
    if (!launched) return err(LGA_ERR_SHAPE, "16-bit GEMM: the launcher refused these arguments");
    return done("lga_op_gemm_splitk");
}

int lga_op_layernorm_fwd(int32_t dtype, const void *x, const float *g, const float *b, void *y, float *mean,
                         float *rstd, int32_t rows, int32_t d, float eps, void *stream) {
    if (!dtype_ok(dtype)) return err(LGA_ERR_ARG, "bad dtype");
    if (rows < 0 || d < 1) return err(LGA_ERR_SHAPE, "bad shape");
    if (!x || !g || !b || !y || !mean || !rstd) return err(LGA_ERR_ARG, "NULL argument");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dtype == LGA_FP32)
        launch_layernorm_fwd<float>(static_cast<const float *>(x), g, b, static_cast<float *>(y), mean, rstd, rows, d, eps, s);
    else
        with16(dtype, [&](auto tag) {
            using E = decltype(tag);
            launch_layernorm_fwd<E>(in16<E>(x), g, b, out16<E>(y), mean, rstd, rows, d, eps, s);
        });
    return done("lga_op_layernorm_fwd");
}

int lga_op_layernorm_bwd(int32_t dtype, const void *dy, const void *x, const float *mean, const float *rstd,
                         const float *g, const void *resid, void *dx, float *dgamma, float *dbeta, float beta,
                         float *scratch, int32_t rows, int32_t d, void *stream) {
    if (!dtype_ok(dtype)) return err(LGA_ERR_ARG, "bad dtype");
    if (rows < 0 || d < 1) return err(LGA_ERR_SHAPE, "bad shape");
    if (!dy || !x || !mean || !rstd || !g || !resid || !dx || !dgamma || !dbeta || !scratch)
        return err(LGA_ERR_ARG, "NULL argument");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dtype == LGA_FP32) {
        launch_layernorm_bwd_dx<float>(static_cast<const float *>(dy), static_cast<const float *>(x), mean, rstd, g,
                                       static_cast<const float *>(resid), static_cast<float *>(dx), rows, d, s, beta, dbeta,
                                       dgamma, scratch);
    } else {
        with16(dtype, [&](auto tag) {
            using E = decltype(tag);
            launch_layernorm_bwd_dx<E>(in16<E>(dy), in16<E>(x), mean, rstd, g, in16<E>(resid), out16<E>(dx), rows, d, s,
                                       beta, dbeta, dgamma, scratch);
        });
    }
    return done("lga_op_layernorm_bwd");
}

uint64_t lga_op_layernorm_bwd_scratch_floats(int32_t rows, int32_t d) {
    if (rows < 0 || d < 0) return 0;
    return layernorm_bwd_partial_floats(rows, d);
}

int lga_op_transpose(const void *in, void *out, int32_t R, int32_t C, int64_t ldi, int64_t ldo, void *stream) {
    if (R < 0 || C < 0 || ldi < C || ldo < R) return err(LGA_ERR_SHAPE, "bad shape");
    if (R % 8 || C % 8 || ldi % 8 || ldo % 8 || !a16(in) || !a16(out))
        return err(LGA_ERR_SHAPE, "transpose needs sizes and leading dimensions that are multiples of 8, 16-byte aligned");
    if ((!in || !out) && R > 0 && C > 0) return err(LGA_ERR_ARG, "NULL argument");
    launch_transpose16(in, out, R, C, ldi, ldo, reinterpret_cast<hipStream_t>(stream));
    return done("lga_op_transpose");
}

int lga_op_transpose_colsum(int32_t dtype, const void *in, void *out, int32_t R, int32_t C, int64_t ldi, int64_t ldo,
                            float beta, float *sums, float *scratch, void *stream) {
    if (dtype != LGA_BF16 && dtype != LGA_FP16) return err(LGA_ERR_ARG, "a 16-bit dtype is needed");
    if (R < 0 || C < 0 || ldi < C || ldo < R) return err(LGA_ERR_SHAPE, "bad shape");
    if (R % 8 || C % 8 || ldi % 8 || ldo % 8 || !a16(in) || !a16(out))
        return err(LGA_ERR_SHAPE, "transpose needs sizes and leading dimensions that are multiples of 8, 16-byte aligned");
    if (((!in || !out) && R > 0 && C > 0) || !sums || !scratch) return err(LGA_ERR_ARG, "NULL argument");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    with16(dtype, [&](auto tag) {
        using E = decltype(tag);
        launch_transpose16_colsum<E>(in16<E>(in), out16<E>(out), R, C, ldi, ldo, beta, sums, scratch, s);
    });
    return done("lga_op_transpose_colsum");
}

uint64_t lga_op_colsum_scratch_floats(int32_t rows, int32_t cols) {
    if (rows < 0 || cols < 0) return 0;
    return colsum_partial_floats(rows, cols);
}

int lga_op_colsum(int32_t dtype, const void *a, int32_t rows, int32_t cols, int32_t ld, float beta, float *out,
                  float *scratch, void *stream) {
    if (!dtype_ok(dtype)) return err(LGA_ERR_ARG, "bad dtype");
    if (rows < 0 || cols < 0 || ld < cols) return err(LGA_ERR_SHAPE, "bad shape");
    if ((!a && rows > 0) || !out || !scratch) return err(LGA_ERR_ARG, "NULL argument");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dtype == LGA_FP32)
        launch_colsum<float>(static_cast<const float *>(a), nullptr, nullptr, nullptr, rows, cols, ld, beta, out, nullptr, scratch, s);
    else
        with16(dtype, [&](auto tag) {
            using E = decltype(tag);
            launch_colsum<E>(in16<E>(a), nullptr, nullptr, nullptr, rows, cols, ld, beta, out, nullptr, scratch, s);
        });
    return done("lga_op_colsum");
}

int lga_op_attention_fwd(int32_t dtype, int32_t kind, const void *qkv, void *out, float *lse, int32_t n_seq,
                         int32_t s_len, int32_t heads, int32_t dh, int32_t causal, void *stream) {
    if (!dtype_ok(dtype) || (kind != 0 && kind != 1)) return err(LGA_ERR_ARG, "bad dtype or kind");
    if (n_seq < 0 || s_len < 1 || heads < 1 || dh < 1) return err(LGA_ERR_SHAPE, "bad shape");
    if ((double)n_seq * heads * ((s_len + 127) / 128) > 2.0e9) return err(LGA_ERR_SHAPE, "sizes overflow the index range");
    if (!qkv || !out || !lse) return err(LGA_ERR_ARG, "NULL argument");
    if (kind == 1 && (!dtype16(dtype) || !attn_bf16_supports(dh) || !a16(qkv) || !a16(out)))
        return err(LGA_ERR_SHAPE, "MFMA attention needs a 16-bit dtype, 16-byte aligned tensors and d_h a multiple of 8 up to 160");
    if (kind == 0 && (size_t)(dh + s_len) * 4 > 60000) return err(LGA_ERR_SHAPE, "sequence too long for the one-wavefront kernel");
    const AttnShape sh{n_seq, s_len, heads, dh, causal != 0};
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dtype == LGA_FP32)
        launch_attn_fwd_simple<float>(static_cast<const float *>(qkv), static_cast<float *>(out), lse, sh, s);
    else
        with16(dtype, [&](auto tag) {
            using E = decltype(tag);
            if (kind == 1) launch_attn_fwd_mfma<E>(in16<E>(qkv), out16<E>(out), lse, sh, s);
            else launch_attn_fwd_simple<E>(in16<E>(qkv), out16<E>(out), lse, sh, s);
        });
    return done("lga_op_attention_fwd");
}

int lga_op_attention_bwd(int32_t dtype, int32_t kind, const void *qkv, const void *out, const float *lse,
                         const void *dout, void *dqkv, float *delta, int32_t n_seq, int32_t s_len, int32_t heads,
                         int32_t dh, int32_t causal, void *stream) {
    if (!dtype_ok(dtype) || (kind != 0 && kind != 1)) return err(LGA_ERR_ARG, "bad dtype or kind");
    if (n_seq < 0 || s_len < 1 || heads < 1 || dh < 1) return err(LGA_ERR_SHAPE, "bad shape");
    if ((double)n_seq * heads * ((s_len + 127) / 128) > 2.0e9) return err(LGA_ERR_SHAPE, "sizes overflow the index range");
    if (!qkv || !out || !lse || !dout || !dqkv || !delta) return err(LGA_ERR_ARG, "NULL argument");
    if (kind == 1 && (!dtype16(dtype) || !attn_bf16_supports(dh) || !a16(qkv) || !a16(out) || !a16(dout) || !a16(dqkv)))
        return err(LGA_ERR_SHAPE, "MFMA attention needs a 16-bit dtype, 16-byte aligned tensors and d_h a multiple of 8 up to 160");
    if (kind == 0 && (size_t)(2 * dh + 2 * s_len) * 4 > 60000) return err(LGA_ERR_SHAPE, "sequence too long for the one-wavefront kernel");
    const AttnShape sh{n_seq, s_len, heads, dh, causal != 0};
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (dtype == LGA_FP32)
        launch_attn_bwd_simple<float>(static_cast<const float *>(qkv), static_cast<const float *>(out), lse,
                                      static_cast<const float *>(dout), static_cast<float *>(dqkv), delta, sh, s);
    else
        with16(dtype, [&](auto tag) {
            using E = decltype(tag);
            if (kind == 1) launch_attn_bwd_mfma<E>(in16<E>(qkv), in16<E>(out), lse, in16<E>(dout), out16<E>(dqkv), delta, sh, s);
            else launch_attn_bwd_simple<E>(in16<E>(qkv), in16<E>(out), lse, in16<E>(dout), out16<E>(dqkv), delta, sh, s);
        });
    return done("lga_op_attention_bwd");
}

uint64_t lga_op_attention_gemm_workspace_bytes(int32_t s_len, int32_t heads) {
    if (s_len < 1 || heads < 1) return 0;
    return attn_gemm_workspace_bytes(s_len, heads);
}

static int check_attention_gemm(int32_t dtype, int32_t n_seq, int32_t s_len, int32_t heads, int32_t dh, const void *ws,
                                uint64_t ws_bytes) {
    if (!dtype16(dtype)) return err(LGA_ERR_ARG, "dtype must be LGA_BF16 or LGA_FP16");
    if (n_seq < 0 || s_len < 1 || heads < 1 || dh < 1) return err(LGA_ERR_SHAPE, "bad shape");
    if (s_len % 8 || dh % 8 || s_len > 32768) return err(LGA_ERR_SHAPE, "GEMM-built attention needs s and d_h to be multiples of 8, s <= 32768");
    if (3.0 * heads * dh > 2.0e9) return err(LGA_ERR_SHAPE, "sizes overflow the index range");
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < attn_gemm_workspace_bytes(s_len, 1))
        return err(LGA_ERR_ARG, "workspace must be 256-byte aligned and hold at least one head (12 s^2 bytes)");
    return LGA_OK;
}

int lga_op_attention_gemm_fwd(int32_t dtype, const void *qkv, void *out, float *lse, int32_t n_seq, int32_t s_len,
                              int32_t heads, int32_t dh, int32_t causal, void *workspace, uint64_t workspace_bytes,
                              void *stream) {
    if (int rc = check_attention_gemm(dtype, n_seq, s_len, heads, dh, workspace, workspace_bytes)) return rc;
    if (!qkv || !out || !lse) return err(LGA_ERR_ARG, "NULL argument");
    if (!a16(qkv) || !a16(out)) return err(LGA_ERR_SHAPE, "GEMM-built attention needs 16-byte aligned tensors");
    const AttnShape sh{n_seq, s_len, heads, dh, causal != 0};
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    with16(dtype, [&](auto tag) {
        using E = decltype(tag);
        launch_attn_fwd_gemm<E>(in16<E>(qkv), out16<E>(out), lse, sh, workspace, workspace_bytes, s);
    });
    return done("lga_op_attention_gemm_fwd");
}

int lga_op_attention_gemm_bwd(int32_t dtype, const void *qkv, const void *out, const float *lse, const void *dout,
                              void *dqkv, float *delta, int32_t n_seq, int32_t s_len, int32_t heads, int32_t dh,
                              int32_t causal, void *workspace, uint64_t workspace_bytes, void *stream) {
    if (int rc = check_attention_gemm(dtype, n_seq, s_len, heads, dh, workspace, workspace_bytes)) return rc;
    if (!qkv || !out || !lse || !dout || !dqkv || !delta) return err(LGA_ERR_ARG, "NULL argument");
    if (!a16(qkv) || !a16(out) || !a16(dout) || !a16(dqkv)) return err(LGA_ERR_SHAPE, "GEMM-built attention needs 16-byte aligned tensors");
    const AttnShape sh{n_seq, s_len, heads, dh, causal != 0};
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    with16(dtype, [&](auto tag) {
        using E = decltype(tag);
        launch_attn_bwd_gemm<E>(in16<E>(qkv), in16<E>(out), lse, in16<E>(dout), out16<E>(dqkv), delta, sh, workspace,
                                workspace_bytes, s);
    });
    return done("lga_op_attention_gemm_bwd");
}

int lga_op_adam(float *w, float *m, float *v, const float *g, void *w16, int32_t w16_dtype, uint64_t n,
                const lga_adam *adam, int32_t *nonfinite, void *stream) {
    if (!adam || (n > 0 && (!w || !m || !v || !g))) return err(LGA_ERR_ARG, "NULL argument");
    if (adam->step < 1) return err(LGA_ERR_STATE, "Adam step t must be >= 1");
    if (w16 && !dtype16(w16_dtype)) return err(LGA_ERR_ARG, "w16_dtype must be LGA_BF16 or LGA_FP16");
    if (!(adam->loss_scale >= 0.f)) return err(LGA_ERR_ARG, "loss_scale must be >= 0");
    if (adam->skip_nonfinite && !nonfinite) return err(LGA_ERR_ARG, "skip_nonfinite needs the nonfinite flag");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    const float grad_mul = (adam->loss_scale > 0.f && adam->loss_scale != 1.f) ? 1.0f / adam->loss_scale : 1.0f;
    int *flag = nullptr;
    if (adam->skip_nonfinite) {
        flag = nonfinite;
        launch_fill_const(reinterpret_cast<float *>(flag), 1, 0.f, s);
        launch_nonfinite_flag(g, n, flag, s);
    }
    with16(w16 ? w16_dtype : LGA_BF16, [&](auto tag) {
        using E = decltype(tag);
        launch_adam<E>(w, m, v, g, out16<E>(w16), n, adam->lr, adam->beta1, adam->beta2, adam->eps, adam->step, grad_mul,
                       flag, s);
    });
    return done("lga_op_adam");
}

}  // extern "C"
