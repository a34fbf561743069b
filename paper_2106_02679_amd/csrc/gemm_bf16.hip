// 16-bit MFMA GEMMs for gfx950, fp32 accumulate: C[M,N] = sum_k A(m,k) B(k,n) + epilogue.
// Every kernel here takes the element type E as its last template argument: bf16 (the default 16-bit mode, from
// which the kernels have their names) or f16 (IEEE half); the two differ in the matrix instruction and in the
// conversions of the epilogues, nothing else.
//
// The three GEMM families of a transformer layer (appendix C.1: each is 2 flop per token per parameter)
//   forward          Y[t,out]  = X[t,in]  W[in,out]
//   input gradient   dX[t,in]  = dY[t,out] W[in,out]^T
//   weight gradient  dW[in,out] (+)= X[t,in]^T dY[t,out]      K = tokens of the micro-batch group
// are all run by the layer stack with BOTH operands k-contiguous (it keeps a transposed 16-bit copy of
// every weight matrix and transposes the two operands of a weight-gradient GEMM beforehand).  That layout
// is served by gemm_bf16_dma_kernel: 256 threads = 4 wavefronts (2x2) on a 256x256x64 tile,
// v_mfma_f32_16x16x32_bf16, tiles moved global -> LDS without passing through registers.
//
// gemm_bf16_kernel is the register-staged predecessor and still serves the other operand layouts of
// the op-level API and the small (128x128-tile) problems: both operands sit in LDS k-contiguous
// (8 chunks of 16 B per row, XOR-swizzled against bank conflicts), so every MFMA operand is one 16-byte
// LDS read; an operand that is not k-contiguous in HBM is transposed in registers (8x8 blocks of 16-bit
// values) on its way from global memory to LDS; two LDS stages; the global loads of tile k+1 are in
// flight while tile k is multiplied.
//
// Common to both: the MFMA is issued with the B tile as its first operand so that each lane ends up with
// 4 consecutive n of one row m (row-major stores of 8 bytes (bf16) or 16 bytes (fp32) per lane, epilogues
// fused); workgroup ids are remapped so that each XCD (ids are dealt round-robin over the 8 XCDs) works on
// a contiguous range of tiles, walked in groups of 8 tile-rows for L2 reuse - or, in the direct-to-LDS kernel on
// tile grids made of whole 16 x 16 blocks, so that all XCDs work on one such block at a time.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <type_traits>

#include "kernels.h"

namespace lga {

namespace {

constexpr int BK = 64;           // k elements per stage

__device__ __forceinline__ int swz(int row) { return ((row >> 1) ^ (row >> 4)) & 7; }

// LDS tile: rows x 64 bf16, row pitch 128 B, chunk c of row r stored at chunk c ^ swz(r).
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * BK + ((chunk ^ swz(row)) << 3); }

// 8x8 transpose of 16-bit values held as 8 rows of 4 dwords.  in[r][q] holds (row r, cols 2q, 2q+1);
// out[c][p] holds (col c, rows 2p, 2p+1).
__device__ __forceinline__ void transpose8x8(const u32x4 (&in)[8], u32x4 (&out)[8]) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t x = in[2 * p][q], y = in[2 * p + 1][q];
            out[2 * q][p] = (x & 0xFFFFu) | (y << 16);
            out[2 * q + 1][p] = (x >> 16) | (y & 0xFFFF0000u);
        }
    }
}

// Global -> register staging of one operand tile (ROWS logical rows x 64 k) through buffer loads.
// The buffer resource is re-based to the tile's (row0, k0) origin for every k tile, so per-lane
// offsets stay small and loop-invariant; a lane whose row or k index is out of range gets an
// offset beyond num_records, for which the hardware returns zeros without touching memory.
//   KMAJOR: storage [rows][ld], k contiguous.  Thread t: chunk t%8, rows t/8 + 32*i.
//   else:   storage [k][ld], row index contiguous.  Thread t owns the 8x8 block with rows
//           8*(t%(ROWS/8)).., k 8*(t/(ROWS/8)).., transposed in registers before the LDS store.
constexpr int kBufRange = 0x40000000;          // 1 GiB window; valid offsets are far below it
constexpr int kBufPoison = 0x7FFFFF00;         // always out of range

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, kBufRange, 0x00020000);
}

template <int ROWS, bool KMAJOR> struct Stager {
    static constexpr int NV = KMAJOR ? ROWS / 32 : 8;
    static constexpr int NOFF = KMAJOR ? NV : 1;
    static_assert(KMAJOR || ROWS <= 256, "one 8x8 block per thread");
    u32x4 v[NV];
    int off[NOFF];       // per-load byte offset inside the tile, or the poison offset for invalid rows
    int ld2;             // leading dimension in bytes

    __device__ __forceinline__ void init(int ld, int row0, int nrows) {
        const int tid = threadIdx.x;
        ld2 = ld * 2;
        if constexpr (KMAJOR) {
            const int voff = (tid >> 3) * ld2 + (tid & 7) * 16;
#pragma unroll
            for (int i = 0; i < NV; ++i) off[i] = (row0 + (tid >> 3) + 32 * i < nrows) ? voff : kBufPoison;
        } else {
            constexpr int CB = ROWS / 8;
            const int r = (tid % CB) * 8, kb = tid / CB;
            off[0] = (tid < ROWS && row0 + r < nrows) ? kb * 8 * ld2 + r * 2 : kBufPoison;
        }
    }

    // base: address of element (row0, k0) of the operand.  Full k tile: no k test.
    __device__ __forceinline__ void load(const void *base) {
        const __amdgpu_buffer_rsrc_t rs = make_rsrc(base);
        if constexpr (KMAJOR) {
#pragma unroll
            for (int i = 0; i < NV; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, off[i], i * 32 * ld2, 0);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, off[0], j * ld2, 0);
        }
    }

    // Last, partial k tile: krem = K - k0 < 64 valid k; the rest reads as zero.
    __device__ __forceinline__ void load_tail(const void *base, int krem) {
        const __amdgpu_buffer_rsrc_t rs = make_rsrc(base);
        const int tid = threadIdx.x;
        if constexpr (KMAJOR) {
            const int kmask = ((tid & 7) * 8 < krem) ? 0 : kBufPoison;     // OR-ing the poison keeps it out of range
#pragma unroll
            for (int i = 0; i < NV; ++i)
                v[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, off[i] | kmask, i * 32 * ld2, 0);
        } else {
            constexpr int CB = ROWS / 8;
            const int kb = tid / CB;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int kmask = (kb * 8 + j < krem) ? 0 : kBufPoison;
                v[j] = __builtin_amdgcn_raw_buffer_load_b128(rs, off[0] | kmask, j * ld2, 0);
            }
        }
    }

    template <class E> __device__ __forceinline__ void store(E *lds) const {
        const int tid = threadIdx.x;
        if constexpr (KMAJOR) {
            const int chunk = tid & 7;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const int r = (tid >> 3) + 32 * i;
                *reinterpret_cast<u32x4 *>(lds + lds_off(r, chunk)) = v[i];
            }
        } else {
            constexpr int CB = ROWS / 8;
            if (ROWS >= 256 || tid < ROWS) {
                u32x4 out[8];
                transpose8x8(v, out);
                const int r = (tid % CB) * 8, kb = tid / CB;
#pragma unroll
                for (int c = 0; c < 8; ++c) *reinterpret_cast<u32x4 *>(lds + lds_off(r + c, kb)) = out[c];
            }
        }
    }
};

template <int EPI, class E>
__device__ __forceinline__ void epilogue4(const GemmParams<E> &p, int m, int n, const float (&a)[4]) {
    const size_t idx = (size_t)m * p.ldc + n;
    if constexpr (EPI == EPI_ACCUM_F32) {
        f32x4 o = {a[0], a[1], a[2], a[3]};
        if (p.beta != 0.f) {
            const f32x4 old = *reinterpret_cast<const f32x4 *>(p.outf + idx);
            o += p.beta * old;
        }
        *reinterpret_cast<f32x4 *>(p.outf + idx) = o;
        return;
    } else {
        float r[4] = {a[0], a[1], a[2], a[3]};
        if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_RESID || EPI == EPI_BIAS_GELU) {
            const f32x4 b = *reinterpret_cast<const f32x4 *>(p.bias + n);
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] += b[i];
        }
        if constexpr (EPI == EPI_BIAS_RESID) {
            const x4<E> x = *reinterpret_cast<const x4<E> *>(p.aux + idx);
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] += (float)x[i];
        }
        if constexpr (EPI == EPI_MUL_DGELU) {
            const x4<E> u = *reinterpret_cast<const x4<E> *>(p.aux + idx);
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] *= gelu_grad_f((float)u[i]);
        }
        if constexpr (EPI == EPI_BIAS_GELU) {
            x4<E> u;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                u[i] = (E)r[i];
                r[i] = gelu_f(r[i]);
            }
            *reinterpret_cast<x4<E> *>(p.out2 + idx) = u;
        }
        x4<E> o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (E)r[i];
        *reinterpret_cast<x4<E> *>(p.out + idx) = o;
    }
}

// The same for 8 consecutive n of one row, with 16-byte accesses (bf16 outputs only): n, ldc multiples of 8 and
// 16-byte aligned tensors.
// aux8: the 8 values of aux at (m, n .. n + 7) for the two epilogues that read it, and b0, b1: the bias of columns
// n .. n + 7 for the three that add it, both loaded by the caller (ahead of time).
template <int EPI, class E>
__device__ __forceinline__ void epilogue8(const GemmParams<E> &p, int m, int n, const f32x4 &lo, const f32x4 &hi,
                                          const x8<E> &aux8, const f32x4 &b0, const f32x4 &b1) {
    static_assert(EPI != EPI_ACCUM_F32, "16-bit outputs only");
    const size_t idx = (size_t)m * p.ldc + n;
    float r[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_RESID || EPI == EPI_BIAS_GELU) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r[i] += b0[i];
            r[4 + i] += b1[i];
        }
    }
    if constexpr (EPI == EPI_BIAS_RESID) {
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] += (float)aux8[i];
    }
    if constexpr (EPI == EPI_MUL_DGELU) {
#pragma unroll
        for (int i = 0; i < 8; ++i) r[i] *= gelu_grad_f((float)aux8[i]);
    }
    if constexpr (EPI == EPI_BIAS_GELU) {
        x8<E> u;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            u[i] = (E)r[i];
            r[i] = gelu_f(r[i]);
        }
        *reinterpret_cast<x8<E> *>(p.out2 + idx) = u;
    }
    x8<E> o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (E)r[i];
    *reinterpret_cast<x8<E> *>(p.out + idx) = o;
}

// Batched launch: work item `tile` belongs to problem tile / ntiles; rebase the operands and outputs onto it.
template <class E> __device__ __forceinline__ void select_problem(GemmParams<E> &p, int &tile, int ntiles) {
    const int z = tile / ntiles;
    tile -= z * ntiles;
    p.A += z * p.strideA;
    p.B += z * p.strideB;
    const long long c = z * p.strideC;
    if (p.out) p.out += c;
    if (p.out2) p.out2 += c;
    if (p.outf) p.outf += c;
    if (p.aux) p.aux += c;
}

template <int BM, int BN, bool A_KM, bool B_KM, int EPI, class E>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmParams<E> p, int tiles_m, int tiles_n) {
    constexpr int WM = BM / 2, WN = BN / 2;     // wavefront tile
    constexpr int FM = WM / 32, FN = WN / 32;   // 32x32 MFMA blocks per wavefront
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    E *lds = reinterpret_cast<E *>(smem_raw);
    // stage s: A at s*(BM+BN)*BK, B right after it
    auto As = [&](int s) { return lds + (size_t)s * (BM + BN) * BK; };
    auto Bs = [&](int s) { return lds + (size_t)s * (BM + BN) * BK + BM * BK; };

    // ---- workgroup -> tile, XCD-aware ----------------------------------------------------
    const int ntiles = tiles_m * tiles_n;
    int tile;
    {
        const int nwork = p.batch > 1 ? ntiles * p.batch : ntiles;      // a batch is ntiles work items per problem
        const int pid = blockIdx.x, xcd = pid & 7, local = pid >> 3;
        const int base = nwork >> 3, rem = nwork & 7;
        tile = xcd * base + (xcd < rem ? xcd : rem) + local;
    }
    if (p.batch > 1) select_problem(p, tile, ntiles);
    constexpr int GROUP_M = 8;
    const int group_size = GROUP_M * tiles_n;
    const int gid = tile / group_size;
    const int first_m = gid * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    const int tm = first_m + (tile % group_size) % gsz;
    const int tn = (tile % group_size) / gsz;
    const int m0 = tm * BM, n0 = tn * BN;
    if (p.tri == 1 && n0 >= m0 + BM) return;             // whole workgroup: the tile lies above the diagonal

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lrow = lane & 31, lhalf = lane >> 5;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    Stager<BM, A_KM> sa;
    Stager<BN, B_KM> sb;
    sa.init(p.lda, m0, p.M);
    sb.init(p.ldb, n0, p.N);
    // element (row0, k) of each operand: k-major rows advance by 1 per k, the others by ld per k
    const E *a_ptr = A_KM ? p.A + (size_t)m0 * p.lda : p.A + m0;
    const E *b_ptr = B_KM ? p.B + (size_t)n0 * p.ldb : p.B + n0;
    const size_t a_step = A_KM ? (size_t)BK : (size_t)BK * p.lda;
    const size_t b_step = B_KM ? (size_t)BK : (size_t)BK * p.ldb;
    if (p.tri == 2) p.K = min(p.K, m0 + BM);
    if (p.tri == 3) {
        const int skip = min(m0, p.K) / BK;              // whole k tiles before the tile's first row
        a_ptr += skip * a_step;
        b_ptr += skip * b_step;
        p.K -= skip * BK;
    }
    const int nk = (p.K + BK - 1) / BK, nk_full = p.K / BK;
    auto load_tile = [&](int t) {
        if (t < nk_full) {
            sa.load(a_ptr + (size_t)t * a_step);
            sb.load(b_ptr + (size_t)t * b_step);
        } else {
            sa.load_tail(a_ptr + (size_t)t * a_step, p.K - t * BK);
            sb.load_tail(b_ptr + (size_t)t * b_step, p.K - t * BK);
        }
    };

    x8<E> af[2][FM], bf[2][FN];
    auto load_frags = [&](int buf, const E *a_lds, const E *b_lds, int ks) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
            af[buf][i] = *reinterpret_cast<const x8<E> *>(a_lds + lds_off(wm * WM + i * 32 + lrow, 2 * ks + lhalf));
#pragma unroll
        for (int j = 0; j < FN; ++j)
            bf[buf][j] = *reinterpret_cast<const x8<E> *>(b_lds + lds_off(wn * WN + j * 32 + lrow, 2 * ks + lhalf));
    };

    load_tile(0);
    sa.store(As(0));
    sb.store(Bs(0));
    __syncthreads();
    load_frags(0, As(0), Bs(0), 0);

    // MFMAs of one k step for accumulator rows [i0, i1) of the wavefront tile
    auto mfma_rows = [&](int fb, int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
                acc[i][j] = mfma_32x32x16<E>(bf[fb][j], af[fb][i], acc[i][j]);
    };
    auto mfma_step = [&](int fb) { mfma_rows(fb, 0, FM); };

    // Instruction-mix hints for the scheduler (masks: 0x008 MFMA, 0x020 VMEM read, 0x100 LDS read,
    // 0x200 LDS write): spread the memory instructions of a k step evenly under its MFMAs.  A CU's
    // texture-address unit takes 16 cycles per 16-byte-per-lane load, so the global loads are
    // issued at no more than one per two MFMAs (64 cycles) per wavefront.
    constexpr int NMF = FM * FN, NDR = FM + FN;
    constexpr int NVA = Stager<BM, A_KM>::NV, NVB = Stager<BN, B_KM>::NV;
    constexpr bool kHints = NMF % NDR == 0 && NMF % NVA == 0 && NMF % NVB == 0 && FM % 2 == 0 &&
                            (NMF / 2) % NDR == 0 && (NVA + NVB) % (NMF / 2) == 0;

    int kt = 0;
    // Main loop: the next k tile exists and is full, so the body is straight-line code.
    //   step 0 : MFMAs | global loads of A(kt+1) | LDS reads of step 1's operands
    //   step 1 : MFMAs | global loads of B(kt+1) | LDS reads of step 2's operands
    //   step 2 : MFMAs | LDS reads of step 3's operands
    //   step 3a: first half of the MFMAs | LDS writes of tile kt+1 into the other stage
    //   barrier
    //   step 3b: second half of the MFMAs | LDS reads of tile kt+1's step-0 operands
    for (; kt + 1 < nk_full; ++kt) {
        const int cur = kt & 1;
        const E *a_lds = As(cur), *b_lds = Bs(cur);
        E *a_nxt = As(cur ^ 1), *b_nxt = Bs(cur ^ 1);

        sa.load(a_ptr + (size_t)(kt + 1) * a_step);
        load_frags(1, a_lds, b_lds, 1);
        mfma_step(0);
        if constexpr (kHints) {
#pragma unroll
            for (int i = 0; i < NMF; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (i % (NMF / NVA) == 0) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                if (i % (NMF / NDR) == 0) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        sb.load(b_ptr + (size_t)(kt + 1) * b_step);
        load_frags(0, a_lds, b_lds, 2);
        mfma_step(1);
        if constexpr (kHints) {
#pragma unroll
            for (int i = 0; i < NMF; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (i % (NMF / NVB) == 0) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                if (i % (NMF / NDR) == 0) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        load_frags(1, a_lds, b_lds, 3);
        mfma_step(0);
        if constexpr (kHints) {
#pragma unroll
            for (int i = 0; i < NDR; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, NMF / NDR, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);

        sa.store(a_nxt);
        sb.store(b_nxt);
        mfma_rows(1, 0, FM / 2);
        if constexpr (kHints) {
#pragma unroll
            for (int i = 0; i < NMF / 2; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x200, (NVA + NVB) / (NMF / 2), 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);

        load_frags(0, a_nxt, b_nxt, 0);
        mfma_rows(1, FM / 2, FM);
        if constexpr (kHints) {
#pragma unroll
            for (int i = 0; i < NDR; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, NMF / 2 / NDR, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    // Remaining tiles (the last full one, and a partial one if K is not a multiple of 64).
    for (; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) load_tile(kt + 1);
        const E *a_lds = As(cur), *b_lds = Bs(cur);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int fb = ks & 1;
            if (ks + 1 < BK / 16) {
                load_frags(fb ^ 1, a_lds, b_lds, ks + 1);
            } else {
                if (more) {
                    sa.store(As(cur ^ 1));
                    sb.store(Bs(cur ^ 1));
                }
                __syncthreads();
                if (more) load_frags(fb ^ 1, As(cur ^ 1), Bs(cur ^ 1), 0);
            }
            mfma_step(fb);
        }
    }

    // ---- epilogue: lane holds row m = lrow, columns n = 8*q + 4*lhalf + (0..3) of each 32x32 block
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int m = m0 + wm * WM + i * 32 + lrow;
        if (m >= p.M) continue;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * WN + j * 32 + 8 * q + 4 * lhalf;
                if (n >= p.N) continue;
                const float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                epilogue4<EPI, E>(p, m, n, v);
            }
        }
    }
}

// ============================================================================================
// Both operands k-contiguous: global -> LDS without passing through registers.
//
// `buffer_load_dwordx4 ... lds` writes lane L's 16 bytes at (LDS base in M0) + 16 L, so one
// wavefront instruction fills 8 consecutive 128-byte tile rows.  The XOR swizzle of the tile is
// obtained on the global side: lane L, which lands in physical chunk L%8 of row r, fetches logical
// chunk (L%8) ^ swz16(r) of that row.  No staging registers, no LDS store instructions, no waits on
// individual loads: the next k tile streams into the other LDS stage while this one is multiplied,
// and one vmcnt wait + barrier per tile publishes it.
//
// The matrix instruction is v_mfma_f32_16x16x32 (a wavefront's 128 x 128 tile = 8 x 8 blocks of 16 x 16, four
// accumulator registers each), not the 32x32x16 one: same flops per cycle and the same LDS operand bytes per k tile,
// twice the 16-bit operand registers read per flop, but a quarter of the fp32 accumulator registers read and written
// per instruction, half per flop (a 16 x 16 block stays in the pipe for 32 k, a 32 x 32 block for 16) - 0.5 instead of
// 0.625 register bytes per multiply-add.  The chip is power-limited on this kernel, and at the board's limit the
// clock it grants is what that difference in power per cycle buys: measured on a merged weight-gradient shape of
// d = 12288 at sustained load and the same 1.35 kW, the 32x32x16 form of this loop ran at 1.50 GHz (1.37 PFLOP/s) and
// this one runs at 1.65 GHz (1.56 PFLOP/s), both with the matrix pipe busy in 0.9 of the cycles.  For the same reason
// the two products that a block receives per k tile are issued back to back (see `half` in the kernel): the second finds
// the accumulator still in the pipe.
__device__ __forceinline__ int swz16(int row) { return (row >> 1) & 7; }      // 16 rows of one chunk column -> 8 chunk places x 2 row parities

template <int BM, int BN, int WGM, int WGN, int EPI, class E>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_dma_kernel(GemmParams<E> p, int tiles_m, int tiles_n) {
    constexpr int NW = WGM * WGN;                   // wavefronts per workgroup, WGM x WGN over the tile
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int FM = WM / 16, FN = WN / 16;       // 16 x 16 blocks of a wavefront's tile
    constexpr int NIA = BM / (8 * NW), NIB = BN / (8 * NW);     // DMA instructions per wavefront per operand tile
    static_assert(BM == BN, "the operand ring below uses one slot size for both operands");
    static_assert(BK == 64, "two k steps of 32 per tile");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    E *lds = reinterpret_cast<E *>(smem_raw);
    // LDS is a ring of kSlots operand tiles of BM x BK.  Operand tiles enter it in the order A(0), B(0), A(1),
    // B(1), ...: A(kt) sits in slot (2 kt) mod kSlots and B(kt) in the next one.  Five slots hold two whole k
    // tiles plus half of a third, which is what lets the loads of A(kt+2) start before tile kt is retired.
    constexpr int kSlots = 5;
    constexpr int kSlotElems = BM * BK;
    auto slot = [&](int q) { return lds + q * kSlotElems; };
    auto wrap = [](int q) { return q >= kSlots ? q - kSlots : q; };

    const int ntiles = tiles_m * tiles_n;
    int tile;
    {
        // with a split k range there are ksplit work items per tile, slice-major
        const int nwork = (EPI == EPI_ACCUM_F32 && p.ksplit > 1) ? ntiles * p.ksplit : p.batch > 1 ? ntiles * p.batch : ntiles;
        const int pid = blockIdx.x, xcd = pid & 7, local = pid >> 3;
        const int base = nwork >> 3, rem = nwork & 7;
        tile = xcd * base + (xcd < rem ? xcd : rem) + local;
    }
    if (p.batch > 1) select_problem(p, tile, ntiles);
    if constexpr (EPI == EPI_ACCUM_F32) {
        if (p.ksplit > 1) {
            // this workgroup multiplies slice z of the k range into partial result z ([M][N], dense)
            const int z = tile / ntiles, k0 = z * p.kchunk;
            tile -= z * ntiles;
            p.A += k0;
            p.B += k0;
            p.K = min(p.K - k0, p.kchunk);
            p.outf = p.partial + (size_t)z * p.M * p.N;
            p.ldc = p.N;
            p.beta = 0.f;
        }
    }
    constexpr int GROUP_M = 8;
    const int group_size = GROUP_M * tiles_n;
    const int gid = tile / group_size;
    const int first_m = gid * GROUP_M;
    const int gsz = min(tiles_m - first_m, GROUP_M);
    int tm = first_m + (tile % group_size) % gsz;
    int tn = (tile % group_size) / gsz;
    if (p.sblock) {
        // Round r of 256 consecutive workgroup ids is one 16 x 16 block of tiles (blocks walk along n first); XCD
        // x = id mod 8 takes rows 8 (x / 4) .. + 7 and columns 4 (x mod 4) .. + 3 of it.  All 8 XCDs then read the
        // same 16 + 16 operand panels at about the same time, so memory sees each of them once per k step instead of
        // once per XCD or per pass over the other dimension; inside an XCD the footprint is the same 8 x 4 tiles.
        const int pid = blockIdx.x, r = pid >> 8, x = pid & 7, local = (pid >> 3) & 31;
        const int nsn = tiles_n >> 4;
        tm = ((r / nsn) << 4) + ((x >> 2) << 3) + (local & 7);
        tn = ((r % nsn) << 4) + ((x & 3) << 2) + (local >> 3);
    }
    const int m0 = tm * BM, n0 = tn * BN;
    if (p.tri == 1 && n0 >= m0 + BM) return;             // whole workgroup: the tile lies above the diagonal

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int l16 = lane & 15, lq = lane >> 4;           // lane = 16 lq + l16

    // A lane's part of a 16 x 16 block: column (m) l16, rows (n) 4 lq .. + 3 - the B tile is the instruction's first
    // operand, so a lane ends with 4 consecutive n of one row m of C.
    f32x4 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Loop-invariant per-lane byte offsets of the DMA loads inside an operand tile (or the poison
    // offset for rows beyond the matrix, which the hardware answers with zeros).
    const int lda2 = p.lda * 2, ldb2 = p.ldb * 2;
    // DMA instruction i of a wavefront fills tile rows [(wave NIA + i) 8, + 8): 1 KB of LDS, right behind that of
    // instruction i - 1.  Four consecutive instructions share one LDS base (M0, a scalar write each time it changes)
    // and tell their places apart by the instruction's immediate offset, 1024 (i % 4) - which the hardware adds to the
    // memory address too, so the per-lane offsets have it subtracted.  (A row is at least 128 bytes long here - the
    // launcher sends shorter leading dimensions to the other kernel - so the difference is never negative.)
    auto dma_row = [&](int i) { return (wave * NIA + i) * 8 + (lane >> 3); };
    static_assert(NIA == NIB && NIA % 4 == 0, "row mapping and M0 groups below");
    int offA[NIA], offB[NIB];
#pragma unroll
    for (int i = 0; i < NIA; ++i) {
        const int r = dma_row(i);
        offA[i] = (m0 + r < p.M) ? r * lda2 + (((lane & 7) ^ swz16(r)) << 4) - (i & 3) * 1024 : kBufPoison;
    }
#pragma unroll
    for (int i = 0; i < NIB; ++i) {
        const int r = dma_row(i);
        offB[i] = (n0 + r < p.N) ? r * ldb2 + (((lane & 7) ^ swz16(r)) << 4) - (i & 3) * 1024 : kBufPoison;
    }
    const E *a_ptr = p.A + (size_t)m0 * p.lda;
    const E *b_ptr = p.B + (size_t)n0 * p.ldb;
    const int nk = (p.K + BK - 1) / BK, nk_full = p.K / BK;

    typedef __attribute__((address_space(3))) void *lds_ptr;
    // One direct-to-LDS load: instruction i of a wavefront's share of an operand tile into ring slot q.  The LDS base
    // is that of the instruction's group of four; the immediate offset (a literal, hence the switch over a value that
    // is a constant wherever this is called) places it inside the group.
    auto lds_dma = [&](const __amdgpu_buffer_rsrc_t &r, int q, int i, int voff, int soff) {
        E *group = slot(q) + (wave * NIA + (i & ~3)) * 8 * BK;
        switch (i & 3) {
            case 0: __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr)group, 16, voff, soff, 0, 0); break;
            case 1: __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr)group, 16, voff, soff, 1024, 0); break;
            case 2: __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr)group, 16, voff, soff, 2048, 0); break;
            default: __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (lds_ptr)group, 16, voff, soff, 3072, 0); break;
        }
    };
    // krem < 64 (partial last tile): k chunks at or beyond krem read as zero.
    auto dma_one = [&](bool is_a, int q, int kt, int krem, int i) {
        const __amdgpu_buffer_rsrc_t r = make_rsrc((is_a ? a_ptr : b_ptr) + (size_t)kt * BK);
        int off = is_a ? offA[i] : offB[i];
        if (krem < BK) off |= ((((lane & 7) ^ swz16(dma_row(i))) * 8 < krem) ? 0 : kBufPoison);
        lds_dma(r, q, i, off, 0);
    };
    // MFMA operands of a whole k tile: block f of k step s (32 k each) of A and of B, 128 registers.  A tile is
    // multiplied in two halves of FM/2 A blocks against all FN B blocks, and the two products of a block - k step 0,
    // k step 1 - are issued one right after the other (see `half` below), so both steps' operands of the blocks in
    // work are in registers at once.  The registers are refilled as they fall free: the A blocks of the second half
    // while the first is multiplied, the next tile's first A half while the second is, and the next tile's B
    // blocks column by column behind the second half's walk over them.  Every LDS read is thus at least 18 block
    // pairs (some 580 cycles) ahead of its use, which rides out the LDS latency spikes that the incoming DMA
    // traffic causes.
    x8<E> af[2][FM], bf[2][FN];
    // LDS byte address of an operand chunk.  A lane reads row (block row 0 + l16), logical chunk 4 s + lq of k step
    // s; the swizzle term of that row is l16 >> 1 whatever the block (blocks start at multiples of 16 rows), so the
    // chunk lies at (lane address) ^ (s << 6) plus a compile-time offset for slot and block.
    static_assert(WM % 16 == 0 && WN % 16 == 0, "whole 16 x 16 blocks");
    const int lane_sw = lq ^ (l16 >> 1);
    const int lane_a = ((wm * WM + l16) * BK + lane_sw * 8) * 2;
    const int lane_b = ((wn * WN + l16) * BK + lane_sw * 8) * 2;
    // operand f of step s (f < FN: B block f, else A block f - FN) of the tile whose A operand is in slot qa
    auto load_frag = [&](int s, int qa, int f) {
        if (f < FN) {
            const int vb = (lane_b ^ (s << 6)) + wrap(qa + 1) * (kSlotElems * 2);
            bf[s][f] = *reinterpret_cast<const x8<E> *>(smem_raw + vb + f * 16 * BK * 2);
        } else {
            const int g = f - FN, va = (lane_a ^ (s << 6)) + qa * (kSlotElems * 2);
            af[s][g] = *reinterpret_cast<const x8<E> *>(smem_raw + va + g * 16 * BK * 2);
        }
    };
    // The same operation for the unrolled main loop, where the ring slot is a compile-time constant.  A wavefront
    // issues strictly in order and, being alone on its SIMD, has nobody to fill the matrix pipe while it issues
    // anything else: measured (32x32x16 form of this loop), 126 other instructions per k tile made a k tile take 2400
    // cycles where its MFMAs need 2048, 64 of them about 2230.  So the loop keeps nothing but the loads themselves:
    //  - LDS operand reads take their address from one of 12 registers set up once - (lane address ^ step term) for
    //    the two steps, in each of the three 64 KB ranges an immediate offset reaches - plus an immediate offset: no
    //    address arithmetic per read;
    //  - the direct-to-LDS loads use one buffer resource per operand for the whole tile and take the k position from
    //    a scalar offset that advances once per k tile; the LDS destination is a constant.
    int pa[2][3], pb[2][3];
#pragma unroll
    for (int v = 0; v < 2; ++v)
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            pa[v][r] = (lane_a ^ (v << 6)) + r * 65536;
            pb[v][r] = (lane_b ^ (v << 6)) + r * 65536;
            // opaque to the compiler, which would otherwise fold the range into each read's offset and add it back
            // with a VALU instruction per read
            asm volatile("" : "+v"(pa[v][r]), "+v"(pb[v][r]));
        }
    auto load_frag_c = [&](int s, int qa, int f) {           // qa: a constant at every call
        const bool is_b = f < FN;
        const int blk = is_b ? f : f - FN;
        const int off = (is_b ? wrap(qa + 1) : qa) * (kSlotElems * 2) + blk * 16 * BK * 2;      // below 160 KB
        const unsigned char *src = smem_raw + (is_b ? pb[s][off >> 16] : pa[s][off >> 16]) + (off & 0xFFFF);
        if (is_b) bf[s][blk] = *reinterpret_cast<const x8<E> *>(src);
        else af[s][blk] = *reinterpret_cast<const x8<E> *>(src);
    };
    const __amdgpu_buffer_rsrc_t rsA = make_rsrc(a_ptr), rsB = make_rsrc(b_ptr);
    // DMA instruction i of a full k tile of A or B into (constant) ring slot q; koff: byte offset of the k tile in a row
    auto dma_c = [&](bool is_a, int q, int koff, int i) {
        // (two calls: the host pass of the compiler does not take a conditional expression of the resource type)
        const int vo = is_a ? offA[i] : offB[i];
        if (is_a) lds_dma(rsA, q, i, vo, koff);
        else lds_dma(rsB, q, i, vo, koff);
    };
    // s_waitcnt immediates (vmcnt in bits 3:0, expcnt 6:4 left at its maximum, lgkmcnt 11:8 = 0): all LDS reads
    // returned and every load landed, or every load but the newest NIA landed.
    constexpr int kWaitVm0 = 0x0070;
    static_assert(NIA < 16, "vmcnt immediate below uses the low four bits only");
    constexpr int kWaitVmA = 0x0070 | NIA;

    // prologue: tile 0 published, tile 1 in flight, tile 0's B blocks and first A half in registers
#pragma unroll
    for (int i = 0; i < NIA; ++i) dma_one(true, 0, 0, p.K, i);
#pragma unroll
    for (int i = 0; i < NIB; ++i) dma_one(false, 1, 0, p.K, i);
    __builtin_amdgcn_s_waitcnt(kWaitVm0);
    __syncthreads();
    if (nk > 1) {
#pragma unroll
        for (int i = 0; i < NIA; ++i) dma_one(true, 2, 1, p.K - BK, i);
#pragma unroll
        for (int i = 0; i < NIB; ++i) dma_one(false, 3, 1, p.K - BK, i);
    }
#pragma unroll
    for (int f = 0; f < FN + FM / 2; ++f) {
        load_frag(0, 0, f);
        load_frag(1, 0, f);
    }

    // Half h of a k tile: A blocks g = 4 h .. 4 h + 3 against all B blocks, column by column (j outer, g inner), and
    // for each block its two products in a row on the same accumulator.  Measured on register operands, a second
    // MFMA on the accumulator of the one just issued costs no cycles and less power than one on another accumulator
    // - the board then grants the clock for it: at the same power, random operands, 2.43 PFLOP/s with strictly
    // adjacent pairs against 2.21 with 64 different accumulators in turn - and in this kernel, on the merged
    // weight-gradient shape of d = 12288 at sustained load, this order gave 1.53 PFLOP/s where the order "all blocks
    // of k step 0, then all of k step 1" gave 1.47 on the same box.
    // Each half also issues its share of the tile's other work, between the pairs and never more than two memory
    // instructions at one place: its 8 direct-to-LDS loads of operand tile `dkt`, one after the first pair of every
    // column; with rd_a, the 8 LDS reads of A blocks ga0 .. ga0 + 3 (both steps) of the tile in slot rqa, after the
    // second and third pair of the first four columns; with rd_b, the two reads of B block j of that tile after the
    // last pair of column j, which was the last use of those registers.
    // The order is pinned (sched_barrier): left to itself the compiler clumps the loads, and a wavefront that issues
    // several in a row right after the barrier, together with the three others, finds the load queue full and
    // stalls with its MFMAs behind it.
    static_assert(NIA == 8 && NIB == 8 && FM == 8 && FN == 8, "one load per column of a half, four A blocks per half");
    // lean_c: the unrolled main loop's forms of the loads (constant slots; dkt is then the k tile's byte offset)
    auto half = [&](auto lean_c, int h, bool do_dma, bool dma_is_a, int dq, int dkt, int dkrem, bool rd_a, int ga0, bool rd_b,
                    int rqa) __attribute__((always_inline)) {
        constexpr bool LEAN = decltype(lean_c)::value;
#pragma unroll
        for (int pr = 0; pr < 4 * FN; ++pr) {
            const int j = pr >> 2, g = 4 * h + (pr & 3);
            mfma_16x16x32_acc<E>(bf[0][j], af[0][g], acc[g][j]);
            mfma_16x16x32_acc<E>(bf[1][j], af[1][g], acc[g][j]);
            if ((pr & 3) == 0 && do_dma) {
                if constexpr (LEAN) dma_c(dma_is_a, dq, dkt, j);
                else dma_one(dma_is_a, dq, dkt, dkrem, j);
            }
            if (rd_a && j < 4 && ((pr & 3) == 1 || (pr & 3) == 2)) {
                const int ia = 2 * j + (pr & 3) - 1;                    // 0 .. 7: block ga0 + ia / 2, step ia % 2
                if constexpr (LEAN) load_frag_c(ia & 1, rqa, FN + ga0 + (ia >> 1));
                else load_frag(ia & 1, rqa, FN + ga0 + (ia >> 1));
            }
            if (rd_b && (pr & 3) == 3) {
                if constexpr (LEAN) {
                    load_frag_c(0, rqa, j);
                    load_frag_c(1, rqa, j);
                } else {
                    load_frag(0, rqa, j);
                    load_frag(1, rqa, j);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // One k tile whose A operand is in ring slot qa; its B blocks and first A half are in registers.  STRAIGHT:
    // tiles kt+1 and kt+2 exist and are full, so nothing is tested.
    //   half 0: MFMAs | LDS reads of this tile's second A half | A(kt+2)'s loads, into the free slot
    //   wait for all loads but A(kt+2)'s + barrier: tile kt+1 is published, and nobody reads tile kt's slots
    //   any more
    //   half 1: MFMAs | LDS reads of tile kt+1's first A half and B blocks | B(kt+2)'s loads, into A(kt)'s slot
    auto k_tile = [&](int kt, int qa, auto straight_c) __attribute__((always_inline)) {
        constexpr bool STRAIGHT = decltype(straight_c)::value;
        const bool more1 = STRAIGHT || kt + 1 < nk, more2 = STRAIGHT || kt + 2 < nk;
        const int krem2 = STRAIGHT ? BK : p.K - (kt + 2) * BK;
        const int qa1 = wrap(qa + 2), qa2 = wrap(qa + 4);      // A(kt+1), A(kt+2); B(kt+2) goes to qa

        half(std::false_type{}, 0, more2, true, qa2, kt + 2, krem2, true, FM / 2, false, qa);
        // A bare s_barrier: __syncthreads() would add a fence that waits for every load, A(kt+2)'s included.
        // The LDS reads above must have returned before other wavefronts may overwrite those slots.
        if (more2)
            __builtin_amdgcn_s_waitcnt(kWaitVmA);
        else
            __builtin_amdgcn_s_waitcnt(kWaitVm0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        half(std::false_type{}, 1, more2, false, qa, kt + 2, krem2, more1, 0, more1, qa1);
    };
    // The same k tile for the unrolled main loop: ring slot qa is a constant, tiles kt+1 and kt+2 exist and are full;
    // koff2 is the byte offset of k tile kt+2 within a row.
    auto k_tile_c = [&](int qa, int koff2) __attribute__((always_inline)) {
        const int qa1 = wrap(qa + 2), qa2 = wrap(qa + 4);
        half(std::true_type{}, 0, true, true, qa2, koff2, BK, true, FM / 2, false, qa);
        __builtin_amdgcn_s_waitcnt(kWaitVmA);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        half(std::true_type{}, 1, true, false, qa, koff2, BK, true, 0, true, qa1);
    };
    int kt = 0, qa = 0;
    // Main loop, unrolled over one period of the ring (five k tiles; the slot of A(kt) is 0, 2, 4, 1, 3, 0, ...).
    {
        int koff2 = 2 * BK * (int)sizeof(E);
        for (; kt + 6 < nk_full; kt += 5) {
            k_tile_c(0, koff2);
            k_tile_c(2, koff2 + 1 * BK * (int)sizeof(E));
            k_tile_c(4, koff2 + 2 * BK * (int)sizeof(E));
            k_tile_c(1, koff2 + 3 * BK * (int)sizeof(E));
            k_tile_c(3, koff2 + 4 * BK * (int)sizeof(E));
            koff2 += 5 * BK * (int)sizeof(E);
        }
    }
    for (; kt + 2 < nk_full; ++kt, qa = wrap(qa + 2)) k_tile(kt, qa, std::true_type{});      // what is left of the full tiles
    for (; kt < nk; ++kt, qa = wrap(qa + 2)) k_tile(kt, qa, std::false_type{});              // the last tiles, with tests
    // the accumulators' last updates must have left the matrix pipe before anything else reads them (see
    // mfma_16x16x32_acc): twice the longest wait the instruction set asks for after a matrix instruction
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");

    if constexpr (EPI != EPI_ACCUM_F32) {
        // bf16 outputs: a lane holds 4 consecutive n of 64 different (row, column group) places, so storing from
        // the accumulators writes 8-byte runs per row and instruction - partial cache lines that reach memory in
        // pieces (measured with the 32 x 32 blocks: up to 2.3 x the output bytes) and scattered reads of the residual /
        // pre-activation.  Instead each wavefront passes its results, 16 rows at a time, through a private piece of
        // the (now idle) operand ring and stores whole rows: 16 lanes x 16 bytes = 256 contiguous bytes, 4 rows per
        // instruction.
        const auto al16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
        const bool wide = ((p.N | p.ldc) & 7) == 0 && al16(p.out) && (EPI != EPI_BIAS_GELU || al16(p.out2)) &&
                          ((EPI != EPI_BIAS_RESID && EPI != EPI_MUL_DGELU) || al16(p.aux)) &&
                          ((EPI != EPI_BIAS && EPI != EPI_BIAS_RESID && EPI != EPI_BIAS_GELU) || al16(p.bias));
        if (wide) {
            constexpr int SP = WN + 4;                                  // staging pitch in floats
            static_assert(NW * 16 * SP * 4 <= 5 * BM * BK * 2, "staging fits in the operand ring");
            // The residual / pre-activation values of the whole wavefront tile are requested first - FM x 4 loads of
            // 16 bytes per lane, into registers the main loop no longer needs - so that their latency is paid once,
            // under the staging of the first strip, and not once per strip.
            constexpr bool kReadsAux = EPI == EPI_BIAS_RESID || EPI == EPI_MUL_DGELU;
            x8<E> aux8[kReadsAux ? FM : 1][kReadsAux ? 4 : 1];
            if constexpr (kReadsAux) {
#pragma unroll
                for (int i = 0; i < FM; ++i)
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const int m = m0 + wm * WM + i * 16 + it * 4 + lq, n = n0 + wn * WN + 8 * l16;
                        if (m < p.M && n < p.N) aux8[i][it] = *reinterpret_cast<const x8<E> *>(p.aux + (size_t)m * p.ldc + n);
                    }
            }
            // A lane stores the same 8 columns of every row: their bias values are read once, not once per store (read
            // inside the loop below, each waits out its whole latency between the staging of two strips: 3 us per tile).
            f32x4 bias_lo = {0.f, 0.f, 0.f, 0.f}, bias_hi = {0.f, 0.f, 0.f, 0.f};
            if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_RESID || EPI == EPI_BIAS_GELU) {
                const int n = n0 + wn * WN + 8 * l16;
                if (n < p.N) {
                    bias_lo = *reinterpret_cast<const f32x4 *>(p.bias + n);
                    bias_hi = *reinterpret_cast<const f32x4 *>(p.bias + n + 4);
                }
            }
            __syncthreads();                                            // every wavefront has left the main loop
            float *stage = reinterpret_cast<float *>(smem_raw) + wave * (16 * SP);
            auto stage_strip = [&](int i) {
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    *reinterpret_cast<f32x4 *>(stage + l16 * SP + j * 16 + 4 * lq) = acc[i][j];
            };
            // LDS operations of one wavefront execute in order, so strip i + 1 may be written into the same piece of
            // LDS as soon as the reads of strip i have been ISSUED: its writes then travel under the wait for those
            // reads.  All eight reads of a strip are issued before any of them is used (left inside the bounds test
            // of its row, each pair waited out the LDS latency on its own: 32 times per tile, 3 us of a tile's 5.5).
            stage_strip(0);
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                asm volatile("" ::: "memory");
                f32x4 lo[4], hi[4];
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    lo[it] = *reinterpret_cast<const f32x4 *>(stage + (it * 4 + lq) * SP + 8 * l16);
                    hi[it] = *reinterpret_cast<const f32x4 *>(stage + (it * 4 + lq) * SP + 8 * l16 + 4);
                }
                asm volatile("" ::: "memory");
                if (i + 1 < FM) stage_strip(i + 1);
                asm volatile("" : "+v"(lo[0]), "+v"(hi[0]), "+v"(lo[1]), "+v"(hi[1]), "+v"(lo[2]), "+v"(hi[2]), "+v"(lo[3]), "+v"(hi[3]));
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int m = m0 + wm * WM + i * 16 + it * 4 + lq, n = n0 + wn * WN + 8 * l16;
                    if (m < p.M && n < p.N)
                        epilogue8<EPI, E>(p, m, n, lo[it], hi[it], aux8[kReadsAux ? i : 0][kReadsAux ? it : 0], bias_lo, bias_hi);
                }
            }
            return;
        }
    }
#pragma unroll
    for (int i = 0; i < FM; ++i) {
        const int m = m0 + wm * WM + i * 16 + l16;
        if (m >= p.M) continue;
#pragma unroll
        for (int j = 0; j < FN; ++j) {
            const int n = n0 + wn * WN + j * 16 + 4 * lq;
            if (n >= p.N) continue;
            const float v[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
            epilogue4<EPI, E>(p, m, n, v);
        }
    }
}

// Explicit instantiations: the host compiler does not always emit the launch stub of a kernel template from its use
// in the launchers below alone.
#define LGA_INSTANTIATE_DMA(EPI)                                                                                 \
    template __global__ void gemm_bf16_dma_kernel<256, 256, 2, 2, EPI, bf16>(GemmParams<bf16>, int, int);        \
    template __global__ void gemm_bf16_dma_kernel<256, 256, 2, 2, EPI, f16>(GemmParams<f16>, int, int)
LGA_INSTANTIATE_DMA(EPI_STORE);
LGA_INSTANTIATE_DMA(EPI_BIAS);
LGA_INSTANTIATE_DMA(EPI_BIAS_RESID);
LGA_INSTANTIATE_DMA(EPI_BIAS_GELU);
LGA_INSTANTIATE_DMA(EPI_MUL_DGELU);
LGA_INSTANTIATE_DMA(EPI_ACCUM_F32);
#undef LGA_INSTANTIATE_DMA

// The kernel that serves a (tile size, layout, epilogue) combination and its dynamic LDS in bytes.
template <int BM, int BN, bool A_KM, bool B_KM, int EPI, class E> struct KernelFor {
    static constexpr bool kDma = A_KM && B_KM && BM == 256;
    static constexpr size_t smem = kDma ? (size_t)5 * BM * BK * sizeof(E)            // the DMA kernel's operand ring
                                        : (size_t)2 * (BM + BN) * BK * sizeof(E);    // two stages of both operands
    static auto get() -> void (*)(GemmParams<E>, int, int) {
        if constexpr (kDma) return gemm_bf16_dma_kernel<BM, BN, 2, 2, EPI, E>;
        else return gemm_bf16_kernel<BM, BN, A_KM, B_KM, EPI, E>;
    }
    // up to 160 KB of dynamic LDS: more than a launch may ask for by default
    static hipError_t raise_lds_limit() {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(get()), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    }
};

template <int BM, int BN, bool A_KM, bool B_KM, int EPI, class E>
void launch_one(const GemmParams<E> &p, hipStream_t s) {
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const size_t smem = KernelFor<BM, BN, A_KM, B_KM, EPI, E>::smem;
    void (*kern)(GemmParams<E>, int, int) = KernelFor<BM, BN, A_KM, B_KM, EPI, E>::get();
    char name[96];
    const char *et = std::is_same<E, bf16>::value ? "bf16" : "f16";       // profile names: gemm_bf16_... or gemm_f16_...
    if (A_KM && B_KM && BM == 256)
        snprintf(name, sizeof(name), "gemm_%s_dma_kernel<%d, %d, %d>", et, BM, BN, EPI);
    else
        snprintf(name, sizeof(name), "gemm_%s_kernel<%d, %d, %s, %s, %d>", et, BM, BN, A_KM ? "true" : "false",
                 B_KM ? "true" : "false", EPI);
    if (p.batch > 1) {                                       // the products of attention: listed apart from the layer's own
        const size_t len = strlen(name);
        snprintf(name + len, sizeof(name) - len, " (batched)");
    }
    const double mn = (double)p.M * p.N;
    const double out_bytes = EPI == EPI_ACCUM_F32 ? (p.beta != 0.f ? 8.0 : 4.0) : (EPI == EPI_BIAS_GELU ? 4.0 : 2.0);
    const double aux_bytes = (EPI == EPI_BIAS_RESID || EPI == EPI_MUL_DGELU) ? 2.0 : 0.0;
    const double nb = p.batch > 1 ? p.batch : 1;
    ProfScope scope(name, nb * 2.0 * mn * p.K,
                    nb * (2.0 * ((double)p.M * p.K + (double)p.K * p.N) + mn * (out_bytes + aux_bytes)), s);
    const int work = tiles_m * tiles_n * (p.ksplit > 1 ? p.ksplit : p.batch > 1 ? p.batch : 1);
    hipLaunchKernelGGL(kern, dim3(work), dim3(256), smem, s, p, tiles_m, tiles_n);
}

// out[m, n] = beta * out[m, n] + sum_z partial[z][m][n]; the slices are added in index order (deterministic).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ partial, int slices, size_t stride,
                                                            float *__restrict__ out, int M, int N, int ldc, float beta) {
    const size_t quads = (size_t)M * (N / 4);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < quads; i += (size_t)gridDim.x * 256) {
        const size_t m = i / (N / 4), n = (i % (N / 4)) * 4;
        f32x4 acc = *reinterpret_cast<const f32x4 *>(partial + m * N + n);
        for (int z = 1; z < slices; ++z) acc += *reinterpret_cast<const f32x4 *>(partial + z * stride + m * N + n);
        float *o = out + m * ldc + n;
        if (beta != 0.f) acc += beta * *reinterpret_cast<const f32x4 *>(o);
        *reinterpret_cast<f32x4 *>(o) = acc;
    }
}

template <bool A_KM, bool B_KM, int EPI, class E> void launch_tiles(const GemmParams<E> &p, hipStream_t s) {
    // Large tiles when they fill the 256 CUs at least about once (the direct-to-LDS kernel is so much faster per
    // tile that a partly idle second round still wins); smaller ones otherwise.
    const long big = (long)((p.M + 255) / 256) * ((p.N + 255) / 256);
    if constexpr (A_KM && B_KM && EPI == EPI_ACCUM_F32) {
        // A weight-gradient GEMM of a narrow layer: few output tiles, very long k.  The k range is cut into slices
        // that run as separate work items of the large-tile kernel and are summed afterwards.
        const int slices = p.batch > 1 ? 1 : gemm_splitk_slices(p.M, p.N, p.K);
        if (slices > 1 && p.partial && (size_t)slices * p.M * p.N <= p.partial_floats && p.N % 4 == 0 && p.ldc % 4 == 0 &&
            (reinterpret_cast<uintptr_t>(p.outf) & 15) == 0) {
            GemmParams<E> q = p;
            q.kchunk = ((p.K + slices - 1) / slices + BK - 1) / BK * BK;
            q.ksplit = (p.K + q.kchunk - 1) / q.kchunk;          // rounding the slice length up may have emptied the last ones
            launch_one<256, 256, A_KM, B_KM, EPI, E>(q, s);
            ProfScope scope("splitk_reduce_kernel", (double)q.ksplit * p.M * p.N,
                            4.0 * p.M * p.N * (q.ksplit + (p.beta != 0.f ? 2.0 : 1.0)), s);
            const size_t quads = (size_t)p.M * (p.N / 4);
            const unsigned blocks = (unsigned)std::min<size_t>((quads + 255) / 256, 256 * 16);
            hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, s, p.partial, q.ksplit, (size_t)p.M * p.N,
                               p.outf, p.M, p.N, p.ldc, p.beta);
            return;
        }
    }
    if (p.batch > 1) {
        // many small problems (the products of attention, one per head): enough work items either way, so take the
        // tile size that pads the output less, the large one on a tie
        const double pad256 = (double)big * 65536.0, pad128 = (double)((p.M + 127) / 128) * ((p.N + 127) / 128) * 16384.0;
        const bool short_rows = A_KM && B_KM && (p.lda < BK || p.ldb < BK);      // see below
        if (big * p.batch >= 128 && pad256 <= 1.15 * pad128 && !short_rows)
            launch_one<256, 256, A_KM, B_KM, EPI, E>(p, s);
        else
            launch_one<128, 128, A_KM, B_KM, EPI, E>(p, s);
        return;
    }
    // (the direct-to-LDS kernel wants rows of at least 128 bytes: see its per-lane load offsets)
    if (big >= 128 && !(A_KM && B_KM && (p.lda < BK || p.ldb < BK))) {
        if constexpr (A_KM && B_KM) {
            const int tm = (p.M + 255) / 256, tn = (p.N + 255) / 256;
            if (tm % 16 == 0 && tn % 16 == 0) {                  // + 1 % on the weight-gradient shapes of d = 12288
                GemmParams<E> q = p;
                q.sblock = 1;
                launch_one<256, 256, A_KM, B_KM, EPI, E>(q, s);
                return;
            }
        }
        launch_one<256, 256, A_KM, B_KM, EPI, E>(p, s);
    } else {
        launch_one<128, 128, A_KM, B_KM, EPI, E>(p, s);
    }
}

}  // namespace

int gemm_splitk_slices(int M, int N, int K) {
    const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
    if (tiles >= 224) return 1;                              // the output alone occupies the chip
    // Work items = tiles x slices run in rounds of 256 (one per CU).  Take the fewest slices (their partial results
    // are written and read again) whose last round is within a tenth of the best filled one.
    long cap = 32;
    if (K > 0) cap = std::min<long>(cap, K / 1024);          // at least 16 k tiles per slice
    cap = std::max<long>(cap, 1);
    auto fill = [&](long s) { return (double)(tiles * s) / (256.0 * ((tiles * s + 255) / 256)); };
    double best = 0.0;
    for (long s = 1; s <= cap; ++s) best = std::max(best, fill(s));
    for (long s = 1; s <= cap; ++s)
        if (fill(s) >= 0.9 * best) return (int)s;
    return 1;
}

bool gemm_mfma_supports(bool a_kmajor, bool b_kmajor, Epilogue epi) {
    if (a_kmajor && !b_kmajor) return epi == EPI_STORE || epi == EPI_BIAS || epi == EPI_BIAS_RESID || epi == EPI_BIAS_GELU;
    if (a_kmajor && b_kmajor) return epi >= EPI_STORE && epi <= EPI_ACCUM_F32;
    if (!a_kmajor && !b_kmajor) return epi == EPI_STORE || epi == EPI_ACCUM_F32;
    return false;
}

template <class E>
bool launch_gemm_mfma(const GemmParams<E> &p, bool a_kmajor, bool b_kmajor, Epilogue epi, hipStream_t s) {
    if (!gemm_mfma_supports(a_kmajor, b_kmajor, epi)) return false;
    // the direct-to-LDS loads address an operand tile's 256 rows with 32-bit byte offsets inside a 1 GiB window
    if (p.lda > kGemmMaxLd || p.ldb > kGemmMaxLd) return false;
    if (p.M == 0 || p.N == 0) return true;
    (void)prepare_kernels();
    // The three operand layouts the layer uses; every epilogue is tied to the family that needs it.
    if (a_kmajor && !b_kmajor) {          // forward
        switch (epi) {
            case EPI_BIAS: launch_tiles<true, false, EPI_BIAS, E>(p, s); break;
            case EPI_BIAS_RESID: launch_tiles<true, false, EPI_BIAS_RESID, E>(p, s); break;
            case EPI_BIAS_GELU: launch_tiles<true, false, EPI_BIAS_GELU, E>(p, s); break;
            default: launch_tiles<true, false, EPI_STORE, E>(p, s); break;
        }
    } else if (a_kmajor && b_kmajor) {    // both operands k-contiguous: the layout the layer stack uses
        switch (epi) {
            case EPI_STORE: launch_tiles<true, true, EPI_STORE, E>(p, s); break;
            case EPI_BIAS: launch_tiles<true, true, EPI_BIAS, E>(p, s); break;
            case EPI_BIAS_RESID: launch_tiles<true, true, EPI_BIAS_RESID, E>(p, s); break;
            case EPI_BIAS_GELU: launch_tiles<true, true, EPI_BIAS_GELU, E>(p, s); break;
            case EPI_MUL_DGELU: launch_tiles<true, true, EPI_MUL_DGELU, E>(p, s); break;
            case EPI_ACCUM_F32: launch_tiles<true, true, EPI_ACCUM_F32, E>(p, s); break;
        }
    } else {                              // weight gradient from operands as stored
        if (epi == EPI_ACCUM_F32) launch_tiles<false, false, EPI_ACCUM_F32, E>(p, s);
        else launch_tiles<false, false, EPI_STORE, E>(p, s);
    }
    return true;
}
template bool launch_gemm_mfma<bf16>(const GemmParams<bf16> &, bool, bool, Epilogue, hipStream_t);
template bool launch_gemm_mfma<f16>(const GemmParams<f16> &, bool, bool, Epilogue, hipStream_t);

namespace {
template <bool A_KM, bool B_KM, int EPI, class E> hipError_t raise_pair() {
    hipError_t e = KernelFor<256, 256, A_KM, B_KM, EPI, E>::raise_lds_limit();
    if (e == hipSuccess) e = KernelFor<128, 128, A_KM, B_KM, EPI, E>::raise_lds_limit();
    return e;
}
template <class E> hipError_t raise_all() {
    hipError_t e = hipSuccess;
    auto next = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    next(raise_pair<true, false, EPI_STORE, E>());
    next(raise_pair<true, false, EPI_BIAS, E>());
    next(raise_pair<true, false, EPI_BIAS_RESID, E>());
    next(raise_pair<true, false, EPI_BIAS_GELU, E>());
    next(raise_pair<true, true, EPI_STORE, E>());
    next(raise_pair<true, true, EPI_BIAS, E>());
    next(raise_pair<true, true, EPI_BIAS_RESID, E>());
    next(raise_pair<true, true, EPI_BIAS_GELU, E>());
    next(raise_pair<true, true, EPI_MUL_DGELU, E>());
    next(raise_pair<true, true, EPI_ACCUM_F32, E>());
    next(raise_pair<false, false, EPI_STORE, E>());
    next(raise_pair<false, false, EPI_ACCUM_F32, E>());
    return e;
}
}  // namespace

hipError_t gemm_prepare_kernels() {
    hipError_t e = raise_all<bf16>();
    if (e == hipSuccess) e = raise_all<f16>();
    return e;
}

}  // namespace lga
