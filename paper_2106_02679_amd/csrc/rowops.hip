// HBM-bound kernels of the layer stack: parameter cast, LayerNorm forward / backward, column
// sums (bias and LayerNorm-affine gradients), Adam, counter-based weight fill.
// All arithmetic is fp32; T (float, bf16 or f16) is only the storage type of activations.
#include <algorithm>

#include "kernels.h"

namespace lga {

namespace {

template <class T> struct VecOf;
template <> struct VecOf<float> { static constexpr int N = 4; };
template <> struct VecOf<bf16> { static constexpr int N = 8; };
template <> struct VecOf<f16> { static constexpr int N = 8; };

template <class T, int N> struct alignas(sizeof(T) * N) Pack { T v[N]; };

template <class T, int N> __device__ __forceinline__ void load_pack(const T *p, float (&out)[N]) {
    if constexpr (N == 1) {
        out[0] = to_f32(p[0]);
    } else {
        const Pack<T, N> t = *reinterpret_cast<const Pack<T, N> *>(p);
#pragma unroll
        for (int i = 0; i < N; ++i) out[i] = to_f32(t.v[i]);
    }
}
template <class T, int N> __device__ __forceinline__ void store_pack(T *p, const float (&in)[N]) {
    if constexpr (N == 1) {
        p[0] = from_f32<T>(in[0]);
    } else {
        Pack<T, N> t;
#pragma unroll
        for (int i = 0; i < N; ++i) t.v[i] = from_f32<T>(in[i]);
        *reinterpret_cast<Pack<T, N> *>(p) = t;
    }
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ------------------------------------------------------------------------------------------
template <class E>
__global__ void cast_kernel(const float *__restrict__ src, E *__restrict__ dst, size_t n, size_t n4) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        const f32x4 v = reinterpret_cast<const f32x4 *>(src)[i];
        x4<E> o;
        o[0] = (E)v[0]; o[1] = (E)v[1]; o[2] = (E)v[2]; o[3] = (E)v[3];
        reinterpret_cast<x4<E> *>(dst)[i] = o;
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = (E)src[i];
}

// *flag = 1 if any of the n values is not finite.  Every thread that sees one stores the same 1 (plain vector store).
__global__ __launch_bounds__(256) void nonfinite_flag_kernel(const float *__restrict__ g, size_t n, size_t n4,
                                                             int *__restrict__ flag) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    bool bad = false;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        const f32x4 v = reinterpret_cast<const f32x4 *>(g)[i];
        // x - x is 0 for finite x and NaN for infinities and NaNs
        const float t = (v[0] - v[0]) + (v[1] - v[1]) + (v[2] - v[2]) + (v[3] - v[3]);
        bad |= !(t == 0.f);
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) bad |= !(g[i] - g[i] == 0.f);
    if (bad) *flag = 1;
}

__global__ void fill_const_kernel(float *dst, size_t n, float value) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = value;
}

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Element i <- std * N(0,1) from a 64-bit mix of (seed, i) and Box-Muller.
__global__ void fill_normal_kernel(float *dst, size_t n, float std, uint64_t seed) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint64_t h = mix64(seed * 0xD1342543DE82EF95ull + i);
        const float u1 = ((float)(uint32_t)(h >> 40) + 1.0f) * (1.0f / 16777217.0f);   // (0, 1)
        const float u2 = (float)(uint32_t)((h >> 8) & 0xFFFFFFu) * (1.0f / 16777216.0f);
        dst[i] = std * sqrtf(-2.0f * __logf(u1)) * __cosf(6.283185307179586f * u2);
    }
}

// ------------------------------------------------------------------------------------------
// LayerNorm forward: one block per row.
template <class T, int V>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(const T *__restrict__ x, const float *__restrict__ g,
                                                            const float *__restrict__ b, T *__restrict__ y,
                                                            float *__restrict__ mean_out, float *__restrict__ rstd_out,
                                                            int d, float eps) {
    __shared__ float red[16];
    const size_t row = blockIdx.x;
    const T *xr = x + row * (size_t)d;
    T *yr = y + row * (size_t)d;
    float s = 0.f;
    for (int c = threadIdx.x * V; c < d; c += blockDim.x * V) {
        float v[V];
        load_pack<T, V>(xr + c, v);
#pragma unroll
        for (int i = 0; i < V; ++i) s += v[i];
    }
    const float mean = block_sum(s, red) / (float)d;
    float q = 0.f;
    for (int c = threadIdx.x * V; c < d; c += blockDim.x * V) {
        float v[V];
        load_pack<T, V>(xr + c, v);
#pragma unroll
        for (int i = 0; i < V; ++i) q += (v[i] - mean) * (v[i] - mean);
    }
    const float var = block_sum(q, red) / (float)d;
    const float rstd = rsqrtf(var + eps);
    if (threadIdx.x == 0) {
        mean_out[row] = mean;
        rstd_out[row] = rstd;
    }
    for (int c = threadIdx.x * V; c < d; c += blockDim.x * V) {
        float v[V], o[V];
        load_pack<T, V>(xr + c, v);
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] = (v[i] - mean) * rstd * g[c + i] + b[c + i];
        store_pack<T, V>(yr + c, o);
    }
}

// The same with a block walking over many rows and everything it needs more than once in registers: each thread
// keeps its NP packs of the row (one global read of x instead of three) and, if CACHE_GB, its gains and biases (read
// per row they are 8 bytes per element of L2 traffic against 4 bytes of x and y).  Wide rows use large blocks, so
// that a thread holds few packs and many wavefronts fit on a CU.  d <= TH * V * NP.  The forward pass and the
// recompute of the backward pass run the same variant, so they still agree bit for bit.
template <class T, int V, int TH, int NP, bool CACHE_GB>
__global__ __launch_bounds__(TH) void layernorm_fwd_rows_kernel(const T *__restrict__ x, const float *__restrict__ g,
                                                                 const float *__restrict__ b, T *__restrict__ y,
                                                                 float *__restrict__ mean_out, float *__restrict__ rstd_out,
                                                                 int rows, int d, float eps) {
    // Two scratch rows used in turn: a sum's barrier also separates the other row's readers from its next writers,
    // so each block-wide sum costs one barrier.
    __shared__ float red[2][16];
    auto sum_all = [&](float v, int which) {
        v = wave_sum(v);
        if ((threadIdx.x & 63) == 0) red[which][threadIdx.x >> 6] = v;
        __syncthreads();
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < TH / 64; ++i) t += red[which][i];
        return t;
    };
    constexpr int NG = CACHE_GB ? NP : 1;
    float gv[NG][V], bv[NG][V];
    if constexpr (CACHE_GB) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) {
#pragma unroll
                for (int q = 0; q < V / 4; ++q) {
                    float t4[4], u4[4];
                    load_pack<float, 4>(g + c + 4 * q, t4);
                    load_pack<float, 4>(b + c + 4 * q, u4);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        gv[p][4 * q + i] = t4[i];
                        bv[p][4 * q + i] = u4[i];
                    }
                }
            }
        }
    }
    // The next row's packs are requested before this row's two block-wide sums, so that loads stay in flight while
    // the block waits at its barriers.
    Pack<T, V> nxt[NP];
    auto request = [&](size_t row) {
        const T *xr = x + row * (size_t)d;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) nxt[p] = *reinterpret_cast<const Pack<T, V> *>(xr + c);
        }
    };
    if (blockIdx.x < (unsigned)rows) request(blockIdx.x);
    for (size_t row = blockIdx.x; row < (size_t)rows; row += gridDim.x) {
        T *yr = y + row * (size_t)d;
        float xv[NP][V];
        float s = 0.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) {
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    xv[p][i] = to_f32(nxt[p].v[i]);
                    s += xv[p][i];
                }
            }
        }
        if (row + gridDim.x < (size_t)rows) request(row + gridDim.x);
        const float mean = sum_all(s, 0) / (float)d;
        float q = 0.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) {
#pragma unroll
                for (int i = 0; i < V; ++i) q += (xv[p][i] - mean) * (xv[p][i] - mean);
            }
        }
        const float var = sum_all(q, 1) / (float)d;
        const float rstd = rsqrtf(var + eps);
        if (threadIdx.x == 0) {
            mean_out[row] = mean;
            rstd_out[row] = rstd;
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) {
                float o[V];
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const float gi = CACHE_GB ? gv[CACHE_GB ? p : 0][i] : g[c + i];
                    const float bi = CACHE_GB ? bv[CACHE_GB ? p : 0][i] : b[c + i];
                    o[i] = (xv[p][i] - mean) * rstd * gi + bi;
                }
                store_pack<T, V>(yr + c, o);
            }
        }
    }
}

// LayerNorm backward w.r.t. the input, plus residual: one block per row.
template <class T, int V>
__global__ __launch_bounds__(256) void layernorm_bwd_dx_kernel(const T *__restrict__ dy, const T *__restrict__ x,
                                                               const float *__restrict__ mean,
                                                               const float *__restrict__ rstd,
                                                               const float *__restrict__ g, const T *resid,
                                                               T *dx, int d) {
    __shared__ float red[16];
    const size_t row = blockIdx.x;
    const T *dyr = dy + row * (size_t)d;
    const T *xr = x + row * (size_t)d;
    const T *rr = resid + row * (size_t)d;
    T *dxr = dx + row * (size_t)d;
    const float mu = mean[row], rs = rstd[row];
    float s1 = 0.f, s2 = 0.f;
    for (int c = threadIdx.x * V; c < d; c += blockDim.x * V) {
        float a[V], v[V];
        load_pack<T, V>(dyr + c, a);
        load_pack<T, V>(xr + c, v);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float gd = a[i] * g[c + i];
            s1 += gd;
            s2 += gd * (v[i] - mu) * rs;
        }
    }
    s1 = block_sum(s1, red) / (float)d;
    s2 = block_sum(s2, red) / (float)d;
    for (int c = threadIdx.x * V; c < d; c += blockDim.x * V) {
        float a[V], v[V], r[V], o[V];
        load_pack<T, V>(dyr + c, a);
        load_pack<T, V>(xr + c, v);
        load_pack<T, V>(rr + c, r);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float xhat = (v[i] - mu) * rs;
            o[i] = r[i] + rs * (a[i] * g[c + i] - s1 - xhat * s2);
        }
        store_pack<T, V>(dxr + c, o);
    }
}

// The same with a block walking over many rows: dy, x and the residual of a row are read once and kept in
// registers, the gains too, the next row is requested before this row's block-wide sums, and the two sums share one
// barrier (two scratch rows used in turn).  d <= TH * V * NP.
// SUMS: every thread also adds up dy and dy * xhat of its columns over the rows its block walks, and the block writes
// them to partial[blockIdx.x][0 / 1][c] - the first pass of the column sums that give the gradients of the LayerNorm
// bias and gain (colsum_final_kernel adds the blocks' rows up in a fixed order), from operands that are in registers anyway.
template <class T, int V, int TH, int NP, bool SUMS>
__global__ __launch_bounds__(TH) void layernorm_bwd_dx_rows_kernel(const T *__restrict__ dy, const T *__restrict__ x,
                                                                   const float *__restrict__ mean,
                                                                   const float *__restrict__ rstd,
                                                                   const float *__restrict__ g, const T *resid, T *dx,
                                                                   int rows, int d, float *__restrict__ partial) {
    __shared__ float red[2][2][16];
    float gv[NP][V];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int c = (p * TH + threadIdx.x) * V;
        if (c < d) {
#pragma unroll
            for (int q = 0; q < V / 4; ++q) {
                float t4[4];
                load_pack<float, 4>(g + c + 4 * q, t4);
#pragma unroll
                for (int i = 0; i < 4; ++i) gv[p][4 * q + i] = t4[i];
            }
        }
    }
    Pack<T, V> na[NP], nx[NP], nr[NP];
    float nmu = 0.f, nrs = 0.f;
    auto request = [&](size_t row) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) {
                na[p] = *reinterpret_cast<const Pack<T, V> *>(dy + row * (size_t)d + c);
                nx[p] = *reinterpret_cast<const Pack<T, V> *>(x + row * (size_t)d + c);
                nr[p] = *reinterpret_cast<const Pack<T, V> *>(resid + row * (size_t)d + c);
            }
        }
        nmu = mean[row];
        nrs = rstd[row];
    };
    float sb[SUMS ? NP : 1][V], sg[SUMS ? NP : 1][V];
#pragma unroll
    for (int p = 0; p < (SUMS ? NP : 1); ++p)
#pragma unroll
        for (int i = 0; i < V; ++i) sb[p][i] = sg[p][i] = 0.f;
    if (blockIdx.x < (unsigned)rows) request(blockIdx.x);
    int turn = 0;
    for (size_t row = blockIdx.x; row < (size_t)rows; row += gridDim.x, turn ^= 1) {
        float gd[NP][V], xh[NP][V], r[NP][V];
        const float rs = nrs, mu = nmu;
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) {
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const float a = to_f32(na[p].v[i]);
                    gd[p][i] = a * gv[p][i];
                    xh[p][i] = (to_f32(nx[p].v[i]) - mu) * rs;
                    r[p][i] = to_f32(nr[p].v[i]);
                    s1 += gd[p][i];
                    s2 += gd[p][i] * xh[p][i];
                    if constexpr (SUMS) {
                        sb[p][i] += a;
                        sg[p][i] += a * xh[p][i];
                    }
                }
            }
        }
        if (row + gridDim.x < (size_t)rows) request(row + gridDim.x);
        s1 = wave_sum(s1);
        s2 = wave_sum(s2);
        if ((threadIdx.x & 63) == 0) {
            red[turn][0][threadIdx.x >> 6] = s1;
            red[turn][1][threadIdx.x >> 6] = s2;
        }
        __syncthreads();
        float t1 = 0.f, t2 = 0.f;
#pragma unroll
        for (int i = 0; i < TH / 64; ++i) {
            t1 += red[turn][0][i];
            t2 += red[turn][1][i];
        }
        t1 /= (float)d;
        t2 /= (float)d;
        T *dxr = dx + row * (size_t)d;
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) {
                float o[V];
#pragma unroll
                for (int i = 0; i < V; ++i) o[i] = r[p][i] + rs * (gd[p][i] - t1 - xh[p][i] * t2);
                store_pack<T, V>(dxr + c, o);
            }
        }
    }
    if constexpr (SUMS) {
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int c = (p * TH + threadIdx.x) * V;
            if (c < d) {
#pragma unroll
                for (int q = 0; q < V / 4; ++q) {       // 16-byte pieces: partial is 16-byte aligned, c a multiple of 4
                    const float b4[4] = {sb[p][4 * q], sb[p][4 * q + 1], sb[p][4 * q + 2], sb[p][4 * q + 3]};
                    const float g4[4] = {sg[p][4 * q], sg[p][4 * q + 1], sg[p][4 * q + 2], sg[p][4 * q + 3]};
                    store_pack<float, 4>(partial + ((size_t)blockIdx.x * 2 + 0) * d + c + 4 * q, b4);
                    store_pack<float, 4>(partial + ((size_t)blockIdx.x * 2 + 1) * d + c + 4 * q, g4);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Column sums, pass 1: block (32 column-threads x 8 row-threads) reduces kColsumRows rows of a
// strip of 32*V columns into partial[row_chunk][2][cols].
constexpr int kColsumRows = 128;

template <class T, int V, bool WITH_XHAT>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T *__restrict__ a, const T *__restrict__ x,
                                                             const float *__restrict__ mean,
                                                             const float *__restrict__ rstd, int rows, int cols,
                                                             int ld, float *__restrict__ partial) {
    __shared__ float red[2][8][32 * V + 1];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c0 = (blockIdx.x * 32 + tx) * V;
    const int r0 = blockIdx.y * kColsumRows;
    const int r1 = min(rows, r0 + kColsumRows);
    float s0[V], s1[V];
#pragma unroll
    for (int i = 0; i < V; ++i) s0[i] = s1[i] = 0.f;
    if (c0 < cols) {
        for (int r = r0 + ty; r < r1; r += 8) {
            float av[V];
            load_pack<T, V>(a + (size_t)r * ld + c0, av);
#pragma unroll
            for (int i = 0; i < V; ++i) s0[i] += av[i];
            if constexpr (WITH_XHAT) {
                float xv[V];
                load_pack<T, V>(x + (size_t)r * ld + c0, xv);
                const float mu = mean[r], rs = rstd[r];
#pragma unroll
                for (int i = 0; i < V; ++i) s1[i] += av[i] * (xv[i] - mu) * rs;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < V; ++i) {
        red[0][ty][tx * V + i] = s0[i];
        red[1][ty][tx * V + i] = s1[i];
    }
    __syncthreads();
    for (int j = threadIdx.x; j < 32 * V; j += 256) {
        const int c = blockIdx.x * 32 * V + j;
        if (c >= cols) continue;
        float t0 = 0.f, t1 = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            t0 += red[0][k][j];
            t1 += red[1][k][j];
        }
        partial[((size_t)blockIdx.y * 2 + 0) * cols + c] = t0;
        if constexpr (WITH_XHAT) partial[((size_t)blockIdx.y * 2 + 1) * cols + c] = t1;
    }
}

// Pass 2: block = 32 columns x 32 groups of row chunks (group q adds chunks q, q + 32, ... in that order), combined
// through LDS in group order, so the result does not depend on scheduling.  Many groups and four loads in flight per
// thread: with the partial rows of a kernel that writes one per block (up to 4096) a thread's chain of dependent adds
// is what this pass takes, not its bytes.
constexpr int kFinalCols = 32, kFinalGroups = 32;

__global__ __launch_bounds__(kFinalCols * kFinalGroups) void colsum_final_kernel(const float *__restrict__ partial, int chunks,
                                                                                 int cols, float beta, float *out0,
                                                                                 float *out1) {
    __shared__ float red[2][kFinalGroups][kFinalCols + 1];
    const int tx = threadIdx.x % kFinalCols, q = threadIdx.x / kFinalCols;
    const int c = blockIdx.x * kFinalCols + tx;
    float t0 = 0.f, t1 = 0.f;
    if (c < cols) {
        int k = q;
        for (; k + 3 * kFinalGroups < chunks; k += 4 * kFinalGroups) {
            float a[4], b[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a[j] = partial[((size_t)(k + j * kFinalGroups) * 2 + 0) * cols + c];
                if (out1) b[j] = partial[((size_t)(k + j * kFinalGroups) * 2 + 1) * cols + c];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                t0 += a[j];
                t1 += b[j];
            }
        }
        for (; k < chunks; k += kFinalGroups) {
            t0 += partial[((size_t)k * 2 + 0) * cols + c];
            if (out1) t1 += partial[((size_t)k * 2 + 1) * cols + c];
        }
    }
    red[0][q][tx] = t0;
    red[1][q][tx] = t1;
    __syncthreads();
    if (q < 2 && c < cols && (q == 0 || out1)) {
        float t = 0.f;
#pragma unroll
        for (int j = 0; j < kFinalGroups; ++j) t += red[q][j][tx];
        float *o = q == 0 ? out0 : out1;
        o[c] = (beta == 0.f ? 0.f : beta * o[c]) + t;
    }
}

// ------------------------------------------------------------------------------------------
// Adam: streams w, m, v, g once (16 B/param in, 12 B + 2 B out).
struct AdamConsts {
    float beta1, beta2, omb1, omb2, inv_bc1, inv_bc2, lr, eps;
    float grad_mul;        // the gradient is multiplied by this first (1 / loss scale; 1 = no scaling, exact)
};

__device__ __forceinline__ void adam_one(float &w, float &m, float &v, float g, const AdamConsts &c) {
    m = c.beta1 * m + c.omb1 * g;
    v = c.beta2 * v + c.omb2 * g * g;
    const float mh = m * c.inv_bc1;
    const float vh = v * c.inv_bc2;
    w = w - c.lr * mh / (sqrtf(vh) + c.eps);
}

template <class E>
__global__ __launch_bounds__(256) void adam_kernel(float *__restrict__ w, float *__restrict__ m,
                                                   float *__restrict__ v, const float *__restrict__ g,
                                                   E *__restrict__ w16, size_t n, size_t n4, AdamConsts c,
                                                   const int *__restrict__ skip) {
    if (skip && *skip) return;          // the gradient held a non-finite value: this update is left out as a whole
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        f32x4 wv = reinterpret_cast<f32x4 *>(w)[i];
        f32x4 mv = reinterpret_cast<f32x4 *>(m)[i];
        f32x4 vv = reinterpret_cast<f32x4 *>(v)[i];
        const f32x4 gv = reinterpret_cast<const f32x4 *>(g)[i];
        float wa[4] = {wv[0], wv[1], wv[2], wv[3]}, ma[4] = {mv[0], mv[1], mv[2], mv[3]};
        float va[4] = {vv[0], vv[1], vv[2], vv[3]};
#pragma unroll
        for (int k = 0; k < 4; ++k) adam_one(wa[k], ma[k], va[k], gv[k] * c.grad_mul, c);
        wv = {wa[0], wa[1], wa[2], wa[3]};
        mv = {ma[0], ma[1], ma[2], ma[3]};
        vv = {va[0], va[1], va[2], va[3]};
        reinterpret_cast<f32x4 *>(w)[i] = wv;
        reinterpret_cast<f32x4 *>(m)[i] = mv;
        reinterpret_cast<f32x4 *>(v)[i] = vv;
        if (w16) {
            x4<E> o;
            o[0] = (E)wa[0]; o[1] = (E)wa[1]; o[2] = (E)wa[2]; o[3] = (E)wa[3];
            reinterpret_cast<x4<E> *>(w16)[i] = o;
        }
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float wa = w[i], ma = m[i], va = v[i];
        adam_one(wa, ma, va, g[i] * c.grad_mul, c);
        w[i] = wa; m[i] = ma; v[i] = va;
        if (w16) w16[i] = (E)wa;
    }
}

// ------------------------------------------------------------------------------------------
// out[c][r] = in[r][c] for 16-bit elements.  A block moves a 128 x 128 tile: each thread loads one
// 8x8 block (16-byte row pieces, lanes along the contiguous direction), transposes it in registers,
// parks it in LDS, and the block then writes whole 256-byte row segments of the output.
constexpr int kTrTile = 128;
constexpr int kTrPitch = kTrTile + 8;     // elements; keeps 16-byte alignment and skews the banks

// SUM: the block also adds up its 128 rows of every column it moves (as values of format E, in fp32) and writes them
// to partial[blockIdx.y][0][c] - the first pass of the column sums (colsum_partial_kernel's layout, same 128-row
// chunks), so that the bias gradient costs no pass of its own over a matrix that is being transposed anyway.
template <class E, bool SUM>
__global__ __launch_bounds__(256) void transpose16_kernel(const uint16_t *__restrict__ in, uint16_t *__restrict__ out,
                                                          int R, int C, long ldi, long ldo, float *__restrict__ partial) {
    static_assert(kTrTile == kColsumRows, "one transposed tile = one chunk of rows of the column sums");
    __shared__ __attribute__((aligned(16))) uint16_t tile[kTrTile * kTrPitch];     // [c][r]
    const int r0 = blockIdx.y * kTrTile, c0 = blockIdx.x * kTrTile;
    const int tid = threadIdx.x;
    {
        const int cb = tid & 15, rb = tid >> 4;           // 16 x 16 blocks of 8 x 8
        u32x4 v[8], t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = r0 + rb * 8 + j, c = c0 + cb * 8;
            v[j] = u32x4{0, 0, 0, 0};
            if (r < R && c < C) v[j] = *reinterpret_cast<const u32x4 *>(in + (size_t)r * ldi + c);
        }
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t x = v[2 * p][q], y = v[2 * p + 1][q];
                t[2 * q][p] = (x & 0xFFFFu) | (y << 16);
                t[2 * q + 1][p] = (x >> 16) | (y & 0xFFFF0000u);
            }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<u32x4 *>(tile + (cb * 8 + i) * kTrPitch + rb * 8) = t[i];
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int c = (tid >> 4) + 16 * j, rch = tid & 15;
        const int gc = c0 + c, gr = r0 + rch * 8;
        const u32x4 piece = *reinterpret_cast<const u32x4 *>(tile + c * kTrPitch + rch * 8);
        if (gc < C && gr < R) *reinterpret_cast<u32x4 *>(out + (size_t)gc * ldo + gr) = piece;
        if constexpr (SUM) {
            // rows beyond R were staged as zeros; the 16 lanes that hold column c's 128 rows are neighbours
            float sum = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t w = piece[q];
                const uint16_t lo = (uint16_t)(w & 0xFFFFu), hi = (uint16_t)(w >> 16);
                sum += to_f32(__builtin_bit_cast(E, lo)) + to_f32(__builtin_bit_cast(E, hi));
            }
#pragma unroll
            for (int m = 8; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, 16);
            if (rch == 0 && gc < C) partial[((size_t)blockIdx.y * 2 + 0) * C + gc] = sum;
        }
    }
}

inline int grid_for(size_t work_items, int block, int max_blocks = 256 * 16) {
    size_t b = (work_items + block - 1) / block;
    if (b < 1) b = 1;
    if (b > (size_t)max_blocks) b = max_blocks;
    return (int)b;
}

}  // namespace

// ==========================================================================================
template <class E> void launch_cast_f32_to_16(const float *src, E *dst, size_t n, hipStream_t s) {
    if (n == 0) return;
    const size_t n4 = (aligned16(src) && (reinterpret_cast<uintptr_t>(dst) & 7u) == 0) ? n / 4 : 0;   // vector part
    ProfScope scope("cast_kernel", 0.0, 6.0 * n, s);
    hipLaunchKernelGGL(cast_kernel<E>, dim3(grid_for(n / 4 + 1, 256)), dim3(256), 0, s, src, dst, n, n4);
}
template void launch_cast_f32_to_16<bf16>(const float *, bf16 *, size_t, hipStream_t);
template void launch_cast_f32_to_16<f16>(const float *, f16 *, size_t, hipStream_t);

void launch_nonfinite_flag(const float *g, size_t n, int *flag, hipStream_t s) {
    if (n == 0) return;
    ProfScope scope("nonfinite_flag_kernel", 0.0, 4.0 * n, s);
    const size_t n4 = aligned16(g) ? n / 4 : 0;
    hipLaunchKernelGGL(nonfinite_flag_kernel, dim3(grid_for(n / 4 + 1, 256, 256 * 8)), dim3(256), 0, s, g, n, n4, flag);
}

void launch_fill_normal(float *dst, size_t n, float std, uint64_t seed, hipStream_t s) {
    if (n == 0) return;
    hipLaunchKernelGGL(fill_normal_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, dst, n, std, seed);
}

void launch_fill_const(float *dst, size_t n, float value, hipStream_t s) {
    if (n == 0) return;
    hipLaunchKernelGGL(fill_const_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, dst, n, value);
}

template <class T>
void launch_layernorm_fwd(const T *x, const float *g, const float *b, T *y, float *mean, float *rstd, int rows,
                          int d, float eps, hipStream_t s) {
    if (rows == 0) return;
    constexpr int V = VecOf<T>::N;
    ProfScope scope("layernorm_fwd_kernel", 8.0 * rows * d, 2.0 * sizeof(T) * rows * (double)d, s);
    // (rows wider than two packs per thread of a 1024-thread block would leave one block per CU: the one-row-per-block
    // kernel, with its many small blocks, is faster there)
    if (d % V == 0 && aligned16(x) && aligned16(y) && aligned16(g) && aligned16(b) && d <= 1024 * V * 2) {
        // rows are dealt to a fixed number of blocks (enough to fill every CU), which keep what they reuse in registers
#define LGA_LN_ROWS(TH, NP) \
        hipLaunchKernelGGL((layernorm_fwd_rows_kernel<T, V, TH, NP, true>), dim3((unsigned)std::min(rows, 256 * (2048 / TH))), \
                           dim3(TH), 0, s, x, g, b, y, mean, rstd, rows, d, eps)
        if (d <= 256 * V) LGA_LN_ROWS(256, 1);
        else if (d <= 512 * V) LGA_LN_ROWS(512, 1);
        else if (d <= 1024 * V) LGA_LN_ROWS(1024, 1);
        else LGA_LN_ROWS(1024, 2);
#undef LGA_LN_ROWS
    } else if (d % V == 0 && aligned16(x) && aligned16(y))
        hipLaunchKernelGGL((layernorm_fwd_kernel<T, V>), dim3(rows), dim3(256), 0, s, x, g, b, y, mean, rstd, d, eps);
    else
        hipLaunchKernelGGL((layernorm_fwd_kernel<T, 1>), dim3(rows), dim3(256), 0, s, x, g, b, y, mean, rstd, d, eps);
}
template void launch_layernorm_fwd<float>(const float *, const float *, const float *, float *, float *, float *, int,
                                          int, float, hipStream_t);
template void launch_layernorm_fwd<bf16>(const bf16 *, const float *, const float *, bf16 *, float *, float *, int,
                                         int, float, hipStream_t);
template void launch_layernorm_fwd<f16>(const f16 *, const float *, const float *, f16 *, float *, float *, int,
                                         int, float, hipStream_t);

// blocks of the row-walking kernel for `rows` rows of length d (0: that kernel does not serve d)
static int lnb_rows_blocks(int rows, int d, int V) {
    if (d > 1024 * V * 2) return 0;
    const int th = d <= 256 * V ? 256 : d <= 512 * V ? 512 : 1024;
    return std::min(rows, 256 * (2048 / th));
}

size_t layernorm_bwd_partial_floats(int rows, int d) {
    // fused sums: one pair of partial rows per block (only widths one pass of the block covers); else the column sums' own
    const size_t fused = (size_t)std::max(lnb_rows_blocks(rows, d, 4), lnb_rows_blocks(rows, d, 8)) * 2 * (size_t)d;
    return std::max(fused, colsum_partial_floats(rows, d));
}

template <class T>
void launch_layernorm_bwd_dx(const T *dy, const T *x, const float *mean, const float *rstd, const float *g,
                             const T *resid, T *dx, int rows, int d, hipStream_t s, float beta, float *dbeta,
                             float *dgamma, float *partial) {
    constexpr int V = VecOf<T>::N;
    const bool sums = dbeta != nullptr;
    const bool vec = d % V == 0 && aligned16(dy) && aligned16(x) && aligned16(resid) && aligned16(dx);
    const bool rows_kernel = vec && aligned16(g) && d <= 1024 * V * 2;
    // the sums ride along where a thread holds one piece of a row (d <= 1024 V): with two, their 4 V extra registers
    // per thread do not fit beside the row
    const bool fused = sums && rows_kernel && d <= 1024 * V && rows > 0 && aligned16(partial);
    if (sums && !fused) launch_colsum<T>(dy, x, mean, rstd, rows, d, d, beta, dbeta, dgamma, partial, s);
    if (rows == 0) return;
    {
        ProfScope scope(fused ? "layernorm_bwd_dx_kernel(with sums)" : "layernorm_bwd_dx_kernel", (fused ? 18.0 : 14.0) * rows * d,
                        4.0 * sizeof(T) * rows * (double)d, s);
        const int blocks = lnb_rows_blocks(rows, d, V);
        if (rows_kernel) {
#define LGA_LNB_ROWS(TH, NP, SUMS) \
            hipLaunchKernelGGL((layernorm_bwd_dx_rows_kernel<T, V, TH, NP, SUMS>), dim3((unsigned)blocks), dim3(TH), 0, s, dy, x, \
                               mean, rstd, g, resid, dx, rows, d, partial)
            if (d <= 256 * V) { if (fused) LGA_LNB_ROWS(256, 1, true); else LGA_LNB_ROWS(256, 1, false); }
            else if (d <= 512 * V) { if (fused) LGA_LNB_ROWS(512, 1, true); else LGA_LNB_ROWS(512, 1, false); }
            else if (d <= 1024 * V) { if (fused) LGA_LNB_ROWS(1024, 1, true); else LGA_LNB_ROWS(1024, 1, false); }
            else LGA_LNB_ROWS(1024, 2, false);
#undef LGA_LNB_ROWS
        } else if (vec)
            hipLaunchKernelGGL((layernorm_bwd_dx_kernel<T, V>), dim3(rows), dim3(256), 0, s, dy, x, mean, rstd, g, resid,
                               dx, d);
        else
            hipLaunchKernelGGL((layernorm_bwd_dx_kernel<T, 1>), dim3(rows), dim3(256), 0, s, dy, x, mean, rstd, g, resid,
                               dx, d);
        if (fused)
            hipLaunchKernelGGL(colsum_final_kernel, dim3((d + kFinalCols - 1) / kFinalCols), dim3(kFinalCols * kFinalGroups), 0, s, partial, blocks, d, beta, dbeta,
                               dgamma);
    }
}
template void launch_layernorm_bwd_dx<float>(const float *, const float *, const float *, const float *,
                                             const float *, const float *, float *, int, int, hipStream_t, float,
                                             float *, float *, float *);
template void launch_layernorm_bwd_dx<bf16>(const bf16 *, const bf16 *, const float *, const float *, const float *,
                                            const bf16 *, bf16 *, int, int, hipStream_t, float, float *, float *, float *);
template void launch_layernorm_bwd_dx<f16>(const f16 *, const f16 *, const float *, const float *, const float *,
                                            const f16 *, f16 *, int, int, hipStream_t, float, float *, float *, float *);

size_t colsum_partial_floats(int rows, int cols) {
    const size_t chunks = ((size_t)rows + kColsumRows - 1) / kColsumRows;
    return (chunks > 0 ? chunks : 1) * 2 * (size_t)cols;
}

template <class T>
void launch_colsum(const T *a, const T *x, const float *mean, const float *rstd, int rows, int cols, int ld,
                   float beta, float *out0, float *out1, float *partial, hipStream_t s, bool timed) {
    if (cols == 0) return;
    constexpr int VMAX = VecOf<T>::N;
    ProfScope scope(out1 ? "colsum_kernels(with xhat)" : "colsum_kernels", (out1 ? 4.0 : 1.0) * rows * cols,
                    (out1 ? 2.0 : 1.0) * sizeof(T) * rows * (double)cols, s, timed);
    const int chunks = rows > 0 ? (rows + kColsumRows - 1) / kColsumRows : 0;
    const bool vec = (cols % VMAX == 0) && (ld % VMAX == 0) && aligned16(a) && (x == nullptr || aligned16(x));
    if (chunks > 0) {
        if (vec) {
            dim3 grid((cols + 32 * VMAX - 1) / (32 * VMAX), chunks);
            if (out1)
                hipLaunchKernelGGL((colsum_partial_kernel<T, VMAX, true>), grid, dim3(256), 0, s, a, x, mean, rstd,
                                   rows, cols, ld, partial);
            else
                hipLaunchKernelGGL((colsum_partial_kernel<T, VMAX, false>), grid, dim3(256), 0, s, a, x, mean, rstd,
                                   rows, cols, ld, partial);
        } else {
            dim3 grid((cols + 31) / 32, chunks);
            if (out1)
                hipLaunchKernelGGL((colsum_partial_kernel<T, 1, true>), grid, dim3(256), 0, s, a, x, mean, rstd, rows,
                                   cols, ld, partial);
            else
                hipLaunchKernelGGL((colsum_partial_kernel<T, 1, false>), grid, dim3(256), 0, s, a, x, mean, rstd, rows,
                                   cols, ld, partial);
        }
    }
    hipLaunchKernelGGL(colsum_final_kernel, dim3((cols + kFinalCols - 1) / kFinalCols), dim3(kFinalCols * kFinalGroups), 0, s, partial, chunks, cols, beta,
                       out0, out1);
}
template void launch_colsum<float>(const float *, const float *, const float *, const float *, int, int, int, float,
                                   float *, float *, float *, hipStream_t, bool);
template void launch_colsum<bf16>(const bf16 *, const bf16 *, const float *, const float *, int, int, int, float,
                                  float *, float *, float *, hipStream_t, bool);
template void launch_colsum<f16>(const f16 *, const f16 *, const float *, const float *, int, int, int, float,
                                  float *, float *, float *, hipStream_t, bool);

void launch_transpose16(const void *in, void *out, int R, int C, long ldi, long ldo, hipStream_t s) {
    if (R == 0 || C == 0) return;
    ProfScope scope("transpose16_kernel", 0.0, 4.0 * R * (double)C, s);
    dim3 grid((C + kTrTile - 1) / kTrTile, (R + kTrTile - 1) / kTrTile);
    hipLaunchKernelGGL((transpose16_kernel<bf16, false>), grid, dim3(256), 0, s, static_cast<const uint16_t *>(in),
                       static_cast<uint16_t *>(out), R, C, ldi, ldo, (float *)nullptr);
}

template <class E>
void launch_transpose16_colsum(const E *in, E *out, int R, int C, long ldi, long ldo, float beta, float *out0,
                               float *partial, hipStream_t s) {
    if (C == 0) return;
    ProfScope scope("transpose16_kernel(with column sums)", 1.0 * R * C, 4.0 * R * (double)C, s);
    const int chunks = (R + kTrTile - 1) / kTrTile;
    if (R > 0) {
        dim3 grid((C + kTrTile - 1) / kTrTile, chunks);
        hipLaunchKernelGGL((transpose16_kernel<E, true>), grid, dim3(256), 0, s, reinterpret_cast<const uint16_t *>(in),
                           reinterpret_cast<uint16_t *>(out), R, C, ldi, ldo, partial);
    }
    hipLaunchKernelGGL(colsum_final_kernel, dim3((C + kFinalCols - 1) / kFinalCols), dim3(kFinalCols * kFinalGroups), 0, s, partial, chunks, C, beta, out0,
                       (float *)nullptr);
}
template void launch_transpose16_colsum<bf16>(const bf16 *, bf16 *, int, int, long, long, float, float *, float *, hipStream_t);
template void launch_transpose16_colsum<f16>(const f16 *, f16 *, int, int, long, long, float, float *, float *, hipStream_t);

template <class E>
void launch_adam(float *w, float *m, float *v, const float *g, E *w16, size_t n, float lr, float beta1, float beta2,
                 float eps, int step, float grad_mul, const int *skip, hipStream_t s) {
    if (n == 0) return;
    AdamConsts c;
    c.beta1 = beta1;
    c.beta2 = beta2;
    c.omb1 = (float)(1.0 - (double)beta1);
    c.omb2 = (float)(1.0 - (double)beta2);
    c.inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    c.inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    c.lr = lr;
    c.eps = eps;
    c.grad_mul = grad_mul;
    ProfScope scope("adam_kernel", 12.0 * n, (w16 ? 30.0 : 28.0) * n, s);
    const bool vec = aligned16(w) && aligned16(m) && aligned16(v) && aligned16(g) &&
                     (reinterpret_cast<uintptr_t>(w16) & 7u) == 0;
    const size_t n4 = vec ? n / 4 : 0;
    hipLaunchKernelGGL(adam_kernel<E>, dim3(grid_for(n / 4 + 1, 256, 256 * 8)), dim3(256), 0, s, w, m, v, g, w16, n, n4,
                       c, skip);
}
template void launch_adam<bf16>(float *, float *, float *, const float *, bf16 *, size_t, float, float, float, float,
                                int, float, const int *, hipStream_t);
template void launch_adam<f16>(float *, float *, float *, const float *, f16 *, size_t, float, float, float, float, int,
                               float, const int *, hipStream_t);

}  // namespace lga
