// Softmax attention for gfx950 on 16-bit tensors (element type E: bf16, or f16 = IEEE half) with fp32 accumulation: forward with an online softmax, and a
// deterministic two-kernel backward (no float atomics).  Causal (decoder: position i sees j <= i) or unmasked
// (encoder: every position sees its whole sequence; only keys past the end of a ragged last tile are masked).
//
// All three kernels are built the same way.  A wavefront owns 32-position blocks of one (sequence, head) and
// lane l owns position l%32 of a block, so every softmax statistic and row sum is lane-local (only the two
// lane halves of a position exchange a value, with one 32-lane swap).  That works because the score tile is
// produced transposed - the tile that is streamed through LDS (keys in the forward and the dQ kernel, queries
// in the dK/dV kernel) is the MFMA's first operand - and the v_mfma_f32_32x32x16 result layout (lane = column,
// 4 consecutive rows per register group) is, after conversion to bf16, directly a valid second operand for the
// next MFMA: its K index is a permutation of the streamed positions, and the first operand of that MFMA is
// read from the streamed tile with the same permutation by the transposing LDS read.  Tiles go from global
// memory straight into LDS (buffer_load ... lds), as stored; nothing is transposed in registers or copied.
//
//   forward      S^T = K Q^T ; P^T = softmax ; O^T += V^T P^T              streams K, V
//   dQ kernel    S^T = K Q^T ; dP^T = V dO^T ; dS^T ; dQ^T += K^T dS^T      streams K, V
//   dK/dV kernel S = Q K^T ; dP = dO V^T ; dV^T += dO^T P ; dK^T += Q^T dS  streams Q, dO
#include <cstdio>
#include <type_traits>

#include "kernels.h"

// The forward kernel's restart loop keeps one requested unroll from being applied in the optimizer's loop pass
// (everything is unrolled later: no array ends up indexed at run time, no scratch memory is used).
#pragma clang diagnostic ignored "-Wpass-failed"

namespace lga {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Second operand straight from global memory: 8 contiguous bf16 of one row (zero if the row is invalid or the
// columns lie beyond the head size dh, a multiple of 8 that may be smaller than the kernel's padded DH).
template <class E> __device__ __forceinline__ x8<E> frag_global(const E *row_ptr, int ks, int half, bool valid, int dh) {
    if (!valid || 16 * ks + 8 * half >= dh) return x8<E>{0, 0, 0, 0, 0, 0, 0, 0};
    return *reinterpret_cast<const x8<E> *>(row_ptr + 16 * ks + 8 * half);
}
// 32x32 fp32 result registers 8*kk .. 8*kk+7 -> 16-bit second operand.
template <class E> __device__ __forceinline__ x8<E> pack16(const f32x16 &v, int kk) {
    x8<E> o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (E)v[8 * kk + e];
    return o;
}

// inside the kernels, whose element type is E
#define MFMA(a, b, c) mfma_32x32x16<E>((a), (b), (c))

// ---- direct-to-LDS tile loads and transposing LDS reads --------------------------------------
// buffer_load_dwordx4 ... lds writes lane L's 16 bytes at (LDS base) + 16 L; rows beyond the sequence get
// an offset outside the buffer's range, which the hardware answers with zeros.
constexpr int kBufRange = 0x40000000;
constexpr int kBufPoison = 0x7FFFFF00;
typedef __attribute__((address_space(3))) void *lds_ptr;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, kBufRange, 0x00020000);
}
// Tiles that are filled by DMA keep their rows at a padded pitch instead of an XOR swizzle, so that every
// MFMA operand address is one per-lane base plus a compile-time offset (swizzled addresses each need
// their own register, and the compiler keeps them all live across the key loop).
//   pitch_rd<DH>  rows read with ds_read_b128 (lane = row): 16 bytes of padding rotate the banks row by row
//   pitch_tr<DH>  rows read with the transposing ds_read_b64_tr_b16, one pass of which covers 4 consecutive
//                 rows x 64 bytes: power-of-two row sizes get 64 bytes of padding, the others already stagger
//   pitch_both<DH> rows read both ways: an odd number of 16-byte slots (ds_read_b128 conflict-free) that is 5 or 13
//                 modulo 16, which leaves the transposing read with two-way conflicts on a few lanes only
template <int DH> constexpr int pitch_rd() { return DH + 8; }
template <int DH> constexpr int pitch_both() { return DH <= 32 ? 40 : DH <= 96 ? 104 : 168; }
template <int DH> constexpr int pitch_tr() { return (DH == 64 || DH == 128) ? DH + 32 : DH; }

// Per-lane part of the address of a transposed operand read from a NATURAL tile [position][pitch]:
// within each group of 16 lanes, lane i passes the address of 4 consecutive values and receives, with lane
// i pointing at (row i/4, columns 4 (i%4) ..+3), column i of rows 0..3.
template <int PITCH> __device__ __forceinline__ int tr_lane_off(int lane) {
    const int i = lane & 15;
    return (4 * (lane >> 5) + (i >> 2)) * PITCH + 16 * ((lane >> 4) & 1) + 4 * (i & 3);
}
// MFMA first operand "row n = 32 c + lrow of the transposed tile, k element e <-> streamed position
// 16 kk + 8 (e/4) + 4 half + e%4" (the permutation that matches a 32x32 MFMA result used as second operand).
// base = tile + tr_lane_off(lane).
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
template <int PITCH, class E> __device__ __forceinline__ x8<E> frag_nat_tr(const E *base, int c, int kk) {
    // Issued as inline assembly: the compiler makes the builtin form wait for every outstanding
    // direct-to-LDS load first (it cannot tell which LDS bytes those write), which would serialise the
    // tile prefetch.  The price: the compiler does not count these reads in lgkmcnt, so wait_tr_reads()
    // must stand between them and their first use.
    const uint32_t addr = (uint32_t)(uintptr_t)base;        // low 32 bits of a generic LDS pointer = LDS address
    u32x2 lo, hi;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "i"((16 * kk * PITCH + 32 * c) * 2));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "i"(((16 * kk + 8) * PITCH + 32 * c) * 2));
    const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(x8<E>, v);
}
// All LDS reads issued so far have returned; the operands listed are tied to the wait so that no use of
// them can be scheduled above it.
template <class V, int N> __device__ __forceinline__ void wait_tr_reads(V (&f)[N]) {
    static_assert(N <= 10, "operand list below");
    if constexpr (N == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]));
    else if constexpr (N == 4) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
    else if constexpr (N == 6)
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]));
    else if constexpr (N == 8)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]));
    else if constexpr (N == 10)
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7]),
                       "+v"(f[8]), "+v"(f[9]));
    else static_assert(N == 2, "unsupported operand count");
}
// DMA of a ROWS x DH tile (global row pitch gp2 bytes) into LDS rows of PITCH elements.  The tile is
// ROWS * (PITCH / 8) slots of 16 bytes, filled 64 at a time; instruction j covers slots [64 j, 64 j + 64).
// Slots that are padding, and rows at or beyond nvalid, get the poison offset (zeros).
template <int ROWS, int DH, int PITCH> struct TileDma {
    static constexpr int SLOTS = PITCH / 8;                 // per row
    static constexpr int NI = (ROWS * SLOTS + 63) / 64;     // instructions that carry data
    static constexpr int NJ = (NI + 3) / 4;                 // per wavefront (4 wavefronts): every wavefront issues NJ,
                                                            // so that "all but the newest tile" is one vmcnt value
    static constexpr int ELEMS = NJ * 4 * 512;              // LDS elements to reserve: 4 NJ instructions of 1 KB
    int row[NJ], off[NJ];
    // dh <= DH: the head size in memory; columns from dh on are padding like the rest of the pitch
    __device__ __forceinline__ void init(int wave, int lane, int gp2, int dh) {
#pragma unroll
        for (int i = 0; i < NJ; ++i) {
            const int slot = (i * 4 + wave) * 64 + lane, r = slot / SLOTS, pc = slot % SLOTS;
            row[i] = (pc < dh / 8 && r < ROWS) ? r : 0x7FFFFFFF;    // padding slots never pass the row test
            off[i] = r * gp2 + (pc << 4);
        }
    }
    // src, dst: tiles of 16-bit elements of either format
    __device__ __forceinline__ void issue(const void *src, void *dst, int nvalid, int wave) const {
        const __amdgpu_buffer_rsrc_t rs = make_rsrc(src);
#pragma unroll
        for (int i = 0; i < NJ; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr)(static_cast<char *>(dst) + (i * 4 + wave) * 1024), 16,
                                                     row[i] < nvalid ? off[i] : kBufPoison, 0, 0, 0);
    }
};

// Workgroup -> ((sequence, head), block rank) for a 1-D grid of n_seq * heads * nblocks workgroups, which the
// hardware hands out in index order.  With the causal mask a (sequence, head)'s blocks differ in length by up to
// the number of blocks: rank is the slow index, so every (sequence, head)'s longest block (rank 0) starts before
// anyone's second longest and the launch ends on the shortest ones.  Without the mask all blocks are equally
// long: rank is the fast index, so the blocks that stream the same keys and values run at the same time and
// share them in the caches.
__device__ __forceinline__ void block_of(const AttnShape &sh, int nblocks, int &bh, int &rank) {
    const int bhs = sh.n_seq * sh.heads;
    if (sh.causal) {
        bh = blockIdx.x % bhs;
        rank = blockIdx.x / bhs;
    } else {
        rank = blockIdx.x % nblocks;
        bh = blockIdx.x / nblocks;
    }
}

// ============================================================================================
// Forward.  One workgroup per (sequence, head, block of 256 queries), see block_of(); rank 0 = the last block.
//
// A wavefront owns 64 queries as two sub-blocks of 32, so every K and V operand it reads from LDS
// feeds two MFMAs; one wavefront per SIMD, with registers for both sub-blocks' output accumulators.
// Key tiles of 64 (K and V as stored, rows of DH) stream from global memory straight into one of two
// LDS stages while the other is multiplied; one barrier per tile publishes it.  V^T operands come from
// the natural V tile through the transposing LDS read.  The online softmax runs per (sub-block, 32 keys).
template <int DH, class E>
__global__ __launch_bounds__(256, 1) void attn_fwd_kernel(const E *__restrict__ qkv, E *__restrict__ out,
                                                       float *__restrict__ lse, AttnShape sh) {
    constexpr int KT = 64;                 // keys per streamed tile
    constexpr int NK = DH / 16, NC = DH / 32;
    constexpr int PK = pitch_rd<DH>(), PV = pitch_tr<DH>();    // LDS row pitches of the K and V tiles
    typedef TileDma<KT, DH, PK> DmaK;
    typedef TileDma<KT, DH, PV> DmaV;
    constexpr int STAGE = DmaK::ELEMS + DmaV::ELEMS;            // elements per stage: K tile, then V tile
    constexpr int NSTAGE = 3;
    constexpr int kWaitOlder = 0x0070 | (DmaK::NJ + DmaV::NJ);  // s_waitcnt lgkmcnt(0) vmcnt(loads of one tile): older tiles landed
    static_assert(DmaK::NJ + DmaV::NJ < 16, "vmcnt immediate uses the low four bits only");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    E *lds = reinterpret_cast<E *>(smem_raw);

    const int qblocks = (sh.s + 255) / 256;
    int bh, rank;
    block_of(sh, qblocks, bh, rank);
    const int qb = qblocks - 1 - rank;
    const int h = bh % sh.heads, b = bh / sh.heads;
    const int dh = sh.dh;                           // head size in memory: a multiple of 8, DH - 24 <= dh <= DH
    const int d = sh.heads * dh;
    const size_t pitch = 3 * (size_t)d;
    const E *seq = qkv + (size_t)b * sh.s * pitch + (size_t)h * dh;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lrow = lane & 31, half = lane >> 5;
    const int qw0 = qb * 256 + wave * 64;          // first query of this wavefront
    const bool causal = sh.causal != 0;
    // Last visible key of sub-block u's lanes = vis_u(u) + vis_lane + 4 half: the query itself, or the end of the sequence.
    const int vis_lane = (causal ? lrow : 0) - 4 * half;
    auto vis_u = [&](int u) { return causal ? qw0 + 32 * u : sh.s - 1; };

    x8<E> qf[2][NK];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int q = qw0 + 32 * u + lrow;
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) qf[u][ks] = frag_global(seq + (size_t)q * pitch, ks, half, q < sh.s, dh);
    }
    // Softmax reference per query, in the log2 domain.  It is FIXED once the query's first 32 keys are seen
    // (p = 2^(score - m_ref) is then exact up to a common factor that the final division removes), so the
    // output accumulators are never rescaled - they live in accumulation registers that only MFMAs touch.
    // A probability far above 1 must still fit the format P is rounded to for the second product - bf16 reaches
    // as far as fp32, IEEE half ends at 65504 - and a probability is never larger than its row's running sum.  So a
    // lane whose sum reaches kSumLimit makes the whole workgroup start over, each query with its reference raised
    // by what its own sum asks for (to a sum of about 2^kTargetLog2), or by kRefStep if the sum overflowed fp32.
    // On ordinary activations bf16 never restarts; half precision does when the keys beyond the first 32 score
    // some 15 (log2 units) higher, which wide layers do reach.  The number of attempts is bounded, so that scores
    // that are infinite or not numbers end in a non-finite output instead of an endless loop.
    constexpr float kSumLimit = std::is_same<E, f16>::value ? 6.0e4f : 1.0e30f;
    constexpr float kRefStep = 64.f, kTargetLog2 = 8.f;
    // Half precision starts 6 units above the best of the first 32 scores: its probabilities then have 22 units of
    // headroom instead of 16, which at the score spread of wide layers saves most restarts, and keys more than 8
    // units below that best score become denormal (still exact to 2^-25 of the row's largest terms).
    constexpr float kRefBias = std::is_same<E, f16>::value ? 6.f : 0.f;
    constexpr int kMaxAttempts = 6;
    f32x16 oacc[2][NC];
    float m_ref[2] = {-INFINITY, -INFINITY}, l_run[2];
    const float c2 = rsqrtf((float)dh) * kLog2e;
    // Plain (not volatile) so that the compiler keeps it an LDS access, which waits for no global load; the
    // barriers' memory clobbers make every read after them a fresh one.
    __shared__ int restart_flag[1];
    if (threadIdx.x == 0) restart_flag[0] = 0;

    // ---- tile loader ------------------------------------------------------------------------
    DmaK dk;
    DmaV dv;
    dk.init(wave, lane, (int)(pitch * 2), dh);
    dv.init(wave, lane, (int)(pitch * 2), dh);
    auto dma_tile = [&](int k0, int stage) {
        E *Ks = lds + stage * STAGE, *Vs = Ks + DmaK::ELEMS;
        dk.issue(seq + (size_t)k0 * pitch + d, Ks, sh.s - k0, wave);
        dv.issue(seq + (size_t)k0 * pitch + 2 * d, Vs, sh.s - k0, wave);
    };
    const int koff = lrow * PK + 8 * half;              // per-lane part of a K operand's address
    const int voff = tr_lane_off<PV>(lane);             // ... and of a V^T operand's

    // ---- one key tile -------------------------------------------------------------------------
    // Four units n = 2 kb + u (key block kb of 32, query sub-block u), each: S = NK MFMAs, the
    // exponentials (VALU), P V = 2 NC MFMAs.  MFMAs of one unit and exponentials of another are
    // independent, so they are issued interleaved - a few MFMAs, then a quarter of a unit's exponentials -
    // and the matrix pipe works under the VALU instructions of the same wavefront:
    //     slot   0      1        2          3          4       5
    //     MFMA   S(0)   S(1)     PV(0) S(2) PV(1) S(3) PV(2)   PV(3)
    //     VALU          exp(0)   exp(1)     exp(2)     exp(3)
    // One set of K operand registers and one of V^T operand registers: the second key block's are read as
    // soon as the first block's last MFMA is issued, under the other work of the slot.  The issue order is
    // pinned (sched_barrier).  With tiles and wavefront query ranges both aligned to 64, a tile is either
    // fully visible or the diagonal one (k0 == qw0), where masked probabilities are forced to zero.
    x8<E> kf[NK], vf[2 * NC], pf[4][2];           // K operands and V^T operands of one key block, P operands [unit]
    f32x16 st[4];                                  // scores per unit
    float pr[2][8];                                // probabilities of half a unit, until they are packed
    auto read_k = [&](const E *Ks, int kb) {
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) kf[ks] = *reinterpret_cast<const x8<E> *>(Ks + kb * 32 * PK + 16 * ks);
    };
    auto read_v = [&](const E *Vs, int kb) {
#pragma unroll
        for (int j2 = 0; j2 < 2; ++j2)
#pragma unroll
            for (int c = 0; c < NC; ++c) vf[j2 * NC + c] = frag_nat_tr<PV>(Vs, c, 2 * kb + j2);
    };
    auto s_group = [&](int n, int g) {             // quarter g of unit n's S MFMAs
        const int u = n & 1;
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            if (ks < g * NK / 4 || ks >= (g + 1) * NK / 4) continue;
            if (ks == 0) {
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                st[n] = MFMA(kf[ks], qf[u][ks], zero);
            } else {
                st[n] = MFMA(kf[ks], qf[u][ks], st[n]);
            }
        }
    };
    auto pv_group = [&](int n, int g) {            // quarter g of unit n's P V MFMAs
        const int u = n & 1;
#pragma unroll
        for (int jc = 0; jc < 2 * NC; ++jc) {
            if (jc < g * 2 * NC / 4 || jc >= (g + 1) * 2 * NC / 4) continue;
            oacc[u][jc % NC] = MFMA(vf[jc], pf[n][jc / NC], oacc[u][jc % NC]);
        }
    };
    // MASKED: probabilities of keys beyond the last visible one are forced to zero (the diagonal part of the
    // sequence, or the ragged last tile of an unmasked sequence); the other copy has no test at all.
    auto exp_group = [&](int n, int g, int k0, auto masked_c) {    // quarter g of unit n's exponentials
        constexpr bool MASKED = decltype(masked_c)::value;
        const int kb = n >> 1, u = n & 1;
        // key of score register r is visible iff 8 (r / 4) + r % 4 <= qrel
        const int qrel = vis_u(u) + vis_lane - (k0 + 32 * kb);
#pragma unroll
        for (int r = 4 * g; r < 4 * g + 4; ++r) {
            float p = __builtin_amdgcn_exp2f(fmaf(st[n][r], c2, -m_ref[u]));
            if (MASKED && 8 * (r >> 2) + (r & 3) > qrel) p = 0.f;
            pr[n & 1][r & 7] = p;           // kept apart from the scores, which sit in accumulation registers
            l_run[u] += p;
        }
        if (g & 1) {
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[n][g >> 1][e] = (E)pr[n & 1][e];
        }
    };
    // No branch inside: with two code paths through the MFMAs the compiler merges their accumulator
    // registers with hundreds of copies per tile.
    auto tile = [&](int k0, int stage, auto masked_c) {
        const E *Ks = lds + stage * STAGE + koff, *Vs = lds + stage * STAGE + DmaK::ELEMS + voff;
        read_k(Ks, 0);
        read_v(Vs, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < 4; ++g) {                  // slot 0: S(0)
            s_group(0, g);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {                  // slot 1: S(1) | exp(0)
            s_group(1, g);
            exp_group(0, g, k0, masked_c);
            __builtin_amdgcn_sched_barrier(0);
        }
        wait_tr_reads(vf);                             // issued at the start of the tile, long since returned
        __builtin_amdgcn_sched_barrier(0);
        read_k(Ks, 1);                                 // the K operand registers are free again: second key block
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < 2; ++n) {                  // slots 2, 3: PV(n) then S(n + 2) | exp(n + 1)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (g < 2) {
                    pv_group(n, 2 * g);
                    pv_group(n, 2 * g + 1);
                } else {
                    s_group(n + 2, 2 * (g - 2));
                    s_group(n + 2, 2 * (g - 2) + 1);
                }
                exp_group(n + 1, g, k0, masked_c);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        read_v(Vs, 1);                                 // ... and so are the V^T operand registers
        __builtin_amdgcn_sched_barrier(0);
        exp_group(3, 0, k0, masked_c);                 // slot 4: exp(3) | PV(2), the reads' latency under exp first
        exp_group(3, 1, k0, masked_c);
        wait_tr_reads(vf);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 2; g < 4; ++g) {
            pv_group(2, 2 * (g - 2));
            pv_group(2, 2 * (g - 2) + 1);
            exp_group(3, g, k0, masked_c);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) pv_group(3, g);    // slot 5: PV(3)
        // overflow guard: a sum this large means that some score was far above the reference
        if (__any(!(l_run[0] < kSumLimit) || !(l_run[1] < kSumLimit))) restart_flag[0] = 1;
    };
    // wait for this wavefront's part of the oldest tile in flight (`newer`: a younger one is in flight too),
    // then a bare s_barrier - a __syncthreads() fence would wait for the younger tile as well.  After it the
    // tile is published and everyone has finished the tile before it, whose stage the next loads overwrite.
    auto publish = [&](bool newer) {
        if (newer)
            __builtin_amdgcn_s_waitcnt(kWaitOlder);
        else
            __builtin_amdgcn_s_waitcnt(0x0070);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    const int kend = causal ? min(sh.s, qb * 256 + 256) : sh.s;      // keys needed by this block: [0, kend)
    const int kfull = causal ? qb * 256 : sh.s / KT * KT;           // tiles before it are fully visible to every wavefront
    for (int attempt = 1;; ++attempt) {
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            l_run[u] = 0.f;
#pragma unroll
            for (int c = 0; c < NC; ++c) oacc[u][c] = zero16;
        }
        // three LDS stages: tile k0 is multiplied while tiles k0 + KT and k0 + 2 KT are in flight
        dma_tile(0, 0);
        if (KT < kend) dma_tile(KT, 1);
        if (attempt == 1) {                  // uniform over the workgroup: the block below holds a barrier
            // First attempt: the scores of each query's first 32 keys fix its softmax reference (key 0 is
            // visible to every query; for the first queries of the sequence these keys are partly masked).
            publish(KT < kend);
            read_k(lds + koff, 0);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                s_group(0, g);
                s_group(1, g);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int qrel = vis_u(u) + vis_lane;
                float raw = -INFINITY;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (8 * (r >> 2) + (r & 3) <= qrel) raw = fmaxf(raw, st[u][r]);
                m_ref[u] = fmaxf(raw, __shfl_xor(raw, 32, 64)) * c2 + kRefBias;
            }
        }
        // No early exit on the restart flag: an attempt that is going to be repeated just runs to its end
        // (rare enough not to matter), which keeps both loops free of side exits - with those the compiler
        // copies the whole output accumulator at every iteration.
        int stage = 0, k0 = 0;
        for (; k0 < kfull; k0 += KT, stage = stage == NSTAGE - 1 ? 0 : stage + 1) {      // fully visible tiles
            publish(true);
            dma_tile(k0 + 2 * KT, stage == 0 ? NSTAGE - 1 : stage - 1);
            tile(k0, stage, std::false_type{});
        }
        for (; k0 < kend; k0 += KT, stage = stage == NSTAGE - 1 ? 0 : stage + 1) {       // the diagonal part
            publish(k0 + KT < kend);
            if (k0 + 2 * KT < kend) dma_tile(k0 + 2 * KT, stage == 0 ? NSTAGE - 1 : stage - 1);
            if (!causal || k0 <= qw0) tile(k0, stage, std::true_type{});
        }
        __syncthreads();
        if (!restart_flag[0] || attempt == kMaxAttempts) break;
        // start over with larger references
        __builtin_amdgcn_s_waitcnt(0x0F70);         // loads of tiles that were still in flight
        __syncthreads();
        if (threadIdx.x == 0) restart_flag[0] = 0;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const float l_tot = l_run[u] + __shfl_xor(l_run[u], 32, 64);      // both lanes of a query see the same sum
            float raise = 0.f;                                                // a query whose sum is fine keeps its reference
            if (!(l_tot < 256.f)) raise = l_tot < 3.0e38f ? ceilf(__log2f(l_tot)) - kTargetLog2 : kRefStep;
            m_ref[u] += raise;
        }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int q = qw0 + 32 * u + lrow;
        const float l_tot = l_run[u] + __shfl_xor(l_run[u], 32, 64);
        if (q < sh.s) {
            const float inv = 1.0f / l_tot;
            E *orow = out + ((size_t)b * sh.s + q) * d + (size_t)h * dh;
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    x4<E> o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o[i] = (E)(oacc[u][c][4 * g + i] * inv);
                    if (c * 32 + 8 * g + 4 * half < dh) *reinterpret_cast<x4<E> *>(orow + c * 32 + 8 * g + 4 * half) = o;
                }
            if (half == 0) lse[((size_t)b * sh.heads + h) * sh.s + q] = m_ref[u] * kLn2 + logf(l_tot);
        }
    }
}

// Explicit instantiations: the host compiler does not always emit the launch stub of a kernel template from its
// use in the launcher below alone.

// ============================================================================================
// delta[b, h, q] = sum_c dO[q, h*dh + c] * O[q, h*dh + c].  out and dout are [tokens][heads * dh]: consecutive
// (token, head) items are consecutive runs of dh elements.  A thread multiplies one 16-byte chunk of each tensor
// (fully coalesced), the chunk sums go through LDS, and one thread per item adds its dh / 8 of them in order.
template <class E>
__global__ __launch_bounds__(256) void attn_delta_kernel(const E *__restrict__ out, const E *__restrict__ dout,
                                                         float *__restrict__ delta, AttnShape sh, int items_per_block) {
    __shared__ float part[256];
    const int cpi = sh.dh / 8;                                            // chunks per item
    const size_t items = (size_t)sh.n_seq * sh.s * sh.heads;
    const size_t item0 = (size_t)blockIdx.x * items_per_block;
    const int tid = threadIdx.x;
    const size_t chunk = item0 * cpi + tid;                               // index into the tensors as arrays of 16-byte chunks
    float acc = 0.f;
    if (tid < items_per_block * cpi && chunk < items * cpi) {
        const x8<E> o = *reinterpret_cast<const x8<E> *>(out + chunk * 8);
        const x8<E> g = *reinterpret_cast<const x8<E> *>(dout + chunk * 8);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc += (float)o[i] * (float)g[i];
    }
    part[tid] = acc;
    __syncthreads();
    if (tid < items_per_block && item0 + tid < items) {
        float t = 0.f;
        for (int c = 0; c < cpi; ++c) t += part[tid * cpi + c];
        const size_t item = item0 + tid;                                  // token * heads + head
        const int h = item % sh.heads;
        const size_t tok = item / sh.heads;
        const size_t bb = tok / sh.s, qq = tok % sh.s;
        delta[(bb * sh.heads + h) * sh.s + qq] = t;
    }
}

// ============================================================================================
// dQ.  One workgroup per (sequence, head, block of 128 queries), see block_of(); rank 0 = the last block.
//
// A wavefront owns 32 queries (Q and dO operands in registers); key tiles of 64 (K and V as stored) stream
// from global memory straight into one of two LDS stages while the other is multiplied, one barrier per
// tile.  K^T operands come from the natural K tile through the transposing LDS read.  Two workgroups per
// CU, so that one's MFMAs run under the other's VALU work.
template <int DH, int OCC, class E>
__global__ __launch_bounds__(256, OCC) void attn_bwd_dq_kernel(const E *__restrict__ qkv, const float *__restrict__ lse,
                                                          const float *__restrict__ delta,
                                                          const E *__restrict__ dout, E *__restrict__ dqkv,
                                                          AttnShape sh) {
    constexpr int KT = 64;
    constexpr int NK = DH / 16, NC = DH / 32;
    constexpr int PK = pitch_both<DH>(), PV = pitch_rd<DH>();
    typedef TileDma<KT, DH, PK> DmaK;
    typedef TileDma<KT, DH, PV> DmaV;
    constexpr int STAGE = DmaK::ELEMS + DmaV::ELEMS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    E *lds = reinterpret_cast<E *>(smem_raw);

    const int qblocks = (sh.s + 127) / 128;
    int bh, rank;
    block_of(sh, qblocks, bh, rank);
    const int qb = qblocks - 1 - rank;
    const int h = bh % sh.heads, b = bh / sh.heads;
    const int dh = sh.dh;                           // head size in memory, <= DH
    const int d = sh.heads * dh;
    const size_t pitch = 3 * (size_t)d;
    const E *seq = qkv + (size_t)b * sh.s * pitch + (size_t)h * dh;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lrow = lane & 31, half = lane >> 5;
    const int qw0 = qb * 128 + wave * 32;
    const int q = qw0 + lrow;
    const bool qvalid = q < sh.s;

    x8<E> qf[NK], dof[NK];
    const E *dorow = dout + ((size_t)b * sh.s + q) * d + (size_t)h * dh;
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
        qf[ks] = frag_global(seq + (size_t)q * pitch, ks, half, qvalid, dh);
        dof[ks] = frag_global(dorow, ks, half, qvalid, dh);
    }
    const size_t stat = ((size_t)b * sh.heads + h) * sh.s + q;
    const float lse2 = qvalid ? lse[stat] * kLog2e : INFINITY;     // invalid rows: p = exp2(-inf) = 0
    const float dl = qvalid ? delta[stat] : 0.f;
    const float scale = rsqrtf((float)dh);
    const float c2 = scale * kLog2e;

    f32x16 acc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;

    DmaK dk;
    DmaV dv;
    dk.init(wave, lane, (int)(pitch * 2), dh);
    dv.init(wave, lane, (int)(pitch * 2), dh);
    auto dma_tile = [&](int k0, int stage) {
        E *Ks = lds + stage * STAGE, *Vs = Ks + DmaK::ELEMS;
        dk.issue(seq + (size_t)k0 * pitch + d, Ks, sh.s - k0, wave);
        dv.issue(seq + (size_t)k0 * pitch + 2 * d, Vs, sh.s - k0, wave);
    };
    const int koff = lrow * PK + 8 * half, voff = lrow * PV + 8 * half;   // per-lane parts of the operand addresses
    const int ktoff = tr_lane_off<PK>(lane);

    const bool causal = sh.causal != 0;
    const int kend = causal ? min(sh.s, qb * 128 + 128) : sh.s;
    dma_tile(0, 0);
    int stage = 0;
    for (int k0 = 0; k0 < kend; k0 += KT, stage ^= 1) {
        // this wavefront's part of tile k0 has landed and its LDS reads of the previous tile have returned; after
        // the barrier the tile is published and the other stage is free for the next one
        __builtin_amdgcn_s_waitcnt(0x0070);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (k0 + KT < kend) dma_tile(k0 + KT, stage ^ 1);
        if (causal && k0 > qw0 + 31) continue;     // whole tile is in this wavefront's future
        const E *Ks = lds + stage * STAGE, *Vs = Ks + DmaK::ELEMS;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const int kbs = k0 + 32 * kb;          // first key of this block of 32
            // in the future of all 32 queries (both are multiples of 32), or past the end of the sequence
            if (causal ? kbs > qw0 : kbs >= sh.s) continue;
            // last visible key of this lane's query, relative to the block: the query itself, or the end of the sequence
            const int klast = causal ? qw0 + lrow - kbs : sh.s - 1 - kbs;
            x8<E> kf[NK], vfr[NK], ktf[2 * NC];
#pragma unroll
            for (int ks = 0; ks < NK; ++ks) {
                kf[ks] = *reinterpret_cast<const x8<E> *>(Ks + koff + kb * 32 * PK + 16 * ks);
                vfr[ks] = *reinterpret_cast<const x8<E> *>(Vs + voff + kb * 32 * PV + 16 * ks);
            }
            f32x16 st, dpt;
#pragma unroll
            for (int ks = 0; ks < NK; ++ks) {
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                st = MFMA(kf[ks], qf[ks], ks == 0 ? zero : st);
                dpt = MFMA(vfr[ks], dof[ks], ks == 0 ? zero : dpt);
            }
            // the K^T operands take over the registers of the K and V operands; their latency passes under the
            // exponentials
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                for (int c = 0; c < NC; ++c) ktf[kk * NC + c] = frag_nat_tr<PK>(Ks + ktoff, c, 2 * kb + kk);
            __builtin_amdgcn_sched_barrier(0);
            if (causal ? kbs == qw0 : kbs + 32 > sh.s) {     // the diagonal block, or the ragged last one: masked keys
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float p = __builtin_amdgcn_exp2f(fmaf(st[r], c2, -lse2));
                    if (8 * (r >> 2) + 4 * half + (r & 3) > klast) p = 0.f;
                    st[r] = p * (dpt[r] - dl);
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) st[r] = __builtin_amdgcn_exp2f(fmaf(st[r], c2, -lse2)) * (dpt[r] - dl);
            }
            wait_tr_reads(ktf);
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const x8<E> dsf = pack16<E>(st, kk);
#pragma unroll
                for (int c = 0; c < NC; ++c) acc[c] = MFMA(ktf[kk * NC + c], dsf, acc[c]);
            }
        }
    }
    if (qvalid) {
        E *orow = dqkv + ((size_t)b * sh.s + q) * pitch + (size_t)h * dh;
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                x4<E> o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = (E)(acc[c][4 * g + i] * scale);
                if (c * 32 + 8 * g + 4 * half < dh) *reinterpret_cast<x4<E> *>(orow + c * 32 + 8 * g + 4 * half) = o;
            }
    }
}


// ============================================================================================
// Tiles that are read both ways - rows with ds_read_b128 and transposed with ds_read_b64_tr_b16 - keep the
// unpadded pitch DH and an XOR swizzle of the 16-byte chunk index that is free of bank conflicts for both:
// 16 consecutive rows put one logical chunk into 16 different bank groups, and 4 consecutive rows (from a
// multiple of 4) put an aligned group of 4 chunks into 4 different ones.
template <int DH> __device__ __forceinline__ int sw_both(int row) {
    if constexpr (DH == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    else if constexpr (DH == 64) return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
    else return (row >> 2) & 3;              // 32, 96, 160: the row pitch already staggers groups of 4 chunks
}
// DMA of a ROWS x DH tile (global row pitch gp2 bytes) into such a tile: lane L of instruction j fills chunk
// slot 64 j + L = row * (DH / 8) + physical chunk, with the logical chunk that the swizzle maps there.
template <int ROWS, int DH> struct TileDmaSw {
    static constexpr int NCH = DH / 8;
    static constexpr int NI = ROWS * NCH / 64;              // instructions per tile
    static constexpr int NJ = (NI + 3) / 4;                 // per wavefront, at most
    static constexpr int ELEMS = ROWS * DH;
    static_assert((ROWS * NCH) % 64 == 0, "tile is a whole number of DMA instructions");
    int row[NJ], off[NJ];
    // dh <= DH: the head size in memory; logical chunks from dh / 8 on are padding (zeros)
    __device__ __forceinline__ void init(int wave, int lane, int gp2, int dh) {
#pragma unroll
        for (int i = 0; i < NJ; ++i) {
            const int slot = (i * 4 + wave) * 64 + lane, r = slot / NCH, pc = slot % NCH;
            row[i] = (pc ^ sw_both<DH>(r)) < dh / 8 ? r : 0x7FFFFFFF;
            off[i] = r * gp2 + ((pc ^ sw_both<DH>(r)) << 4);
        }
    }
    // src, dst: tiles of 16-bit elements of either format
    __device__ __forceinline__ void issue(const void *src, void *dst, int nvalid, int wave) const {
        const __amdgpu_buffer_rsrc_t rs = make_rsrc(src);
#pragma unroll
        for (int i = 0; i < NJ; ++i) {
            const int j = i * 4 + wave;
            if (j >= NI) continue;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr)(static_cast<char *>(dst) + j * 1024), 16, row[i] < nvalid ? off[i] : kBufPoison,
                                                     0, 0, 0);
        }
    }
};
// Per-lane address parts (elements) of the two kinds of operand read from such a tile.  The swizzle splits
// into a part that XORs the chunk group (DH = 64, 128 only) and one that XORs within the group, which leaves
// few distinct lane values; everything else is a compile-time offset.
template <int DH> struct BothAddr {
    static constexpr int NG = DH == 128 ? 4 : DH == 64 ? 2 : 1;     // chunk groups the swizzle permutes
    int nb[NG][2];      // natural read: [chunk group][ks & 1]
    int tb[NG][2];      // transposed read: [32-column block c (if NG > 1)][second half of the 16 positions]
    __device__ __forceinline__ void init(int lane) {
        const int lrow = lane & 31, half = lane >> 5, i = lane & 15, g = (lane >> 4) & 1;
        const int s = sw_both<DH>(lrow), s_hi = s >> 2, s_lo = s & 3;
#pragma unroll
        for (int a = 0; a < NG; ++a)
#pragma unroll
            for (int e = 0; e < 2; ++e) nb[a][e] = lrow * DH + 32 * (a ^ s_hi) + (((2 * e + half) ^ s_lo) << 3);
#pragma unroll
        for (int sec = 0; sec < 2; ++sec) {
            const int row = 8 * sec + 4 * half + (i >> 2);           // + 16 kk, which does not change the swizzle
            const int t = sw_both<DH>(row), t_hi = t >> 2, t_lo = t & 3;
            const int b = 2 * g + ((i & 3) >> 1);
#pragma unroll
            for (int c = 0; c < NG; ++c) tb[c][sec] = row * DH + 32 * (c ^ t_hi) + ((b ^ t_lo) << 3) + 4 * (i & 1);
        }
    }
    // MFMA first operand: row 32 u + lrow of the tile, k = 16 ks + 8 half + (0..7)
    template <class E> __device__ __forceinline__ x8<E> nat(const E *tile, int u, int ks) const {
        const int a = ks >> 1;
        return *reinterpret_cast<const x8<E> *>(tile + 32 * u * DH + nb[NG > 1 ? a : 0][ks & 1] + (NG > 1 ? 0 : 32 * a));
    }
    // MFMA first operand "row 32 c + lrow of the transposed tile, k element e <-> tile row 16 kk + 8 (e/4) + 4 half + e%4"
    template <class E> __device__ __forceinline__ x8<E> tr(const E *tile, int c, int kk) const {
        const uint32_t a0 = (uint32_t)(uintptr_t)(tile + tb[NG > 1 ? c : 0][0]);
        const uint32_t a1 = (uint32_t)(uintptr_t)(tile + tb[NG > 1 ? c : 0][1]);
        u32x2 lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(a0), "i"((16 * kk * DH + (NG > 1 ? 0 : 32 * c)) * 2));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a1), "i"((16 * kk * DH + (NG > 1 ? 0 : 32 * c)) * 2));
        const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
        return __builtin_bit_cast(x8<E>, v);
    }
};

// ============================================================================================
// dK, dV.  One workgroup per (sequence, head, block of 128 keys), see block_of(); rank = key block index (with the
// causal mask the first key block has the most queries).
//
// A wavefront owns 32 keys (K and V operands in registers, dK and dV accumulators); query tiles of 64 (Q and
// dO as stored) stream from global memory straight into one of three LDS stages, one barrier per tile.  Every
// tile is read both ways: rows for S = Q K^T and dP = dO V^T, transposed for dV^T += dO^T P and dK^T += Q^T dS.
// With the causal mask the first two query tiles of a key block contain its diagonal (masked, partly skipped); all
// later ones - without the mask, all tiles from the start of the sequence - are fully visible and go through a loop
// without tests (rows past the end of the sequence are zero and carry zero statistics: they add nothing).
template <int DH, class E>
__global__ __launch_bounds__(256, 1) void attn_bwd_dkv_kernel(const E *__restrict__ qkv, const float *__restrict__ lse,
                                                              const float *__restrict__ delta,
                                                              const E *__restrict__ dout, E *__restrict__ dqkv,
                                                              AttnShape sh) {
    constexpr int QT = 64, NST = 3;
    constexpr int NK = DH / 16, NC = DH / 32;
    typedef TileDmaSw<QT, DH> Dma;
    constexpr int TILE = Dma::ELEMS, STAGE = 2 * TILE;          // Q tile, then dO tile
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    E *lds = reinterpret_cast<E *>(smem_raw);
    float *lse_s = reinterpret_cast<float *>(lds + NST * STAGE);     // [NST][QT]  log-sum-exp, log2 domain, negated
    float *dl_s = lse_s + NST * QT;                                  // [NST][QT]  delta

    int bh, kb128;
    block_of(sh, (sh.s + 127) / 128, bh, kb128);
    const int h = bh % sh.heads, b = bh / sh.heads;
    const int dh = sh.dh;                           // head size in memory, <= DH
    const int d = sh.heads * dh;
    const size_t pitch = 3 * (size_t)d;
    const E *seq = qkv + (size_t)b * sh.s * pitch + (size_t)h * dh;
    const E *doseq = dout + (size_t)b * sh.s * d + (size_t)h * dh;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lrow = lane & 31, half = lane >> 5;
    const int kw0 = kb128 * 128 + wave * 32;        // first key of this wavefront
    const int key = kw0 + lrow;
    const bool kvalid = key < sh.s;

    x8<E> kf[NK], vf[NK];
#pragma unroll
    for (int ks = 0; ks < NK; ++ks) {
        kf[ks] = frag_global(seq + (size_t)key * pitch + d, ks, half, kvalid, dh);
        vf[ks] = frag_global(seq + (size_t)key * pitch + 2 * d, ks, half, kvalid, dh);
    }
    const float scale = rsqrtf((float)dh);
    const float c2 = scale * kLog2e;
    const size_t stat0 = ((size_t)b * sh.heads + h) * sh.s;

    f32x16 dk[NC], dv[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) dk[c][r] = dv[c][r] = 0.f;

    Dma dq_, do_;
    dq_.init(wave, lane, (int)(pitch * 2), dh);
    do_.init(wave, lane, d * 2, dh);
    BothAddr<DH> ad;
    ad.init(lane);
    const bool causal = sh.causal != 0;
    // Tile t holds queries [qbeg + 64 t, +64); with the causal mask, queries before the key block see none of its keys.  Its row statistics go through registers: wavefront 0 fetches the
    // log-sum-exps, wavefront 1 the deltas, one tile ahead of the tile data, and they are stored to LDS before
    // the barrier that publishes the tile.
    const int qbeg = causal ? kb128 * 128 : 0;
    const int ntiles = (sh.s - qbeg + QT - 1) / QT;
    auto dma_tile = [&](int t, int stage) {
        const int q0 = qbeg + QT * t;
        dq_.issue(seq + (size_t)q0 * pitch, lds + stage * STAGE, sh.s - q0, wave);
        do_.issue(doseq + (size_t)q0 * d, lds + stage * STAGE + TILE, sh.s - q0, wave);
    };
    auto load_stat = [&](int t) -> float {
        const int qq = qbeg + QT * t + lane;
        if (wave == 0) return qq < sh.s ? -lse[stat0 + qq] * kLog2e : 0.f;
        if (wave == 1) return qq < sh.s ? delta[stat0 + qq] : 0.f;
        return 0.f;
    };
    auto store_stat = [&](int stage, float v) {
        if (wave == 0) lse_s[stage * QT + lane] = v;
        if (wave == 1) dl_s[stage * QT + lane] = v;
    };

    // one (32 keys x 32 queries) unit of tile `stage`: query rows [32 u, 32 u + 32) of the tile, first query qs
    auto unit = [&](int stage, int u, int qs, auto masked_c) {
        constexpr bool MASKED = decltype(masked_c)::value;
        const E *Qs = lds + stage * STAGE, *dOs = Qs + TILE;
        x8<E> qn[NK], don[NK];
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            qn[ks] = ad.nat(Qs, u, ks);
            don[ks] = ad.nat(dOs, u, ks);
        }
        f32x4 l4[4], d4[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            l4[g] = *reinterpret_cast<const f32x4 *>(lse_s + stage * QT + 32 * u + 8 * g + 4 * half);
            d4[g] = *reinterpret_cast<const f32x4 *>(dl_s + stage * QT + 32 * u + 8 * g + 4 * half);
        }
        f32x16 s_, dp;
#pragma unroll
        for (int ks = 0; ks < NK; ++ks) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            s_ = MFMA(qn[ks], kf[ks], ks == 0 ? zero : s_);
            dp = MFMA(don[ks], vf[ks], ks == 0 ? zero : dp);
        }
        // the transposed operands take over the registers of the row operands; their latency passes under the
        // exponentials
        __builtin_amdgcn_sched_barrier(0);
        x8<E> dot[2 * NC], qt[2 * NC];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                dot[kk * NC + c] = ad.tr(dOs, c, 2 * u + kk);
                qt[kk * NC + c] = ad.tr(Qs, c, 2 * u + kk);
            }
        __builtin_amdgcn_sched_barrier(0);
        f32x16 pr;
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = 4 * g + i;
                float p = __builtin_amdgcn_exp2f(fmaf(s_[r], c2, l4[g][i]));
                if (MASKED && qs + 8 * g + 4 * half + i < key) p = 0.f;
                pr[r] = p;
                s_[r] = p * (dp[r] - d4[g][i]);
            }
        x8<E> pf[2], dsf[2];
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            pf[kk] = pack16<E>(pr, kk);
            dsf[kk] = pack16<E>(s_, kk);
        }
        wait_tr_reads(dot);
        wait_tr_reads(qt);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                dv[c] = MFMA(dot[kk * NC + c], pf[kk], dv[c]);
                dk[c] = MFMA(qt[kk * NC + c], dsf[kk], dk[c]);
            }
    };
    // wait for this wavefront's part of the oldest tile in flight (`newer`: a younger one is in flight too),
    // then a bare s_barrier - a __syncthreads() fence would wait for the younger tile as well
    constexpr int kLoadsPerTile = 2 * Dma::NJ;      // upper bound of what a wavefront issues per tile
    static_assert(Dma::NI % 4 == 0 && kLoadsPerTile < 16, "every wavefront issues the same number of loads per tile");
    auto publish = [&](bool newer) {
        if (newer)
            __builtin_amdgcn_s_waitcnt(0x0070 | kLoadsPerTile);
        else
            __builtin_amdgcn_s_waitcnt(0x0070);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // tile t is multiplied while tiles t + 1 and t + 2 are in flight
    float stat = load_stat(0);
    dma_tile(0, 0);
    store_stat(0, stat);
    if (ntiles > 1) {
        stat = load_stat(1);
        dma_tile(1, 1);
    }
    // start of every iteration: tile t + 1's statistics go to LDS (published by the barrier after next... by
    // the next iteration's barrier), tile t is published, tile t + 2 is requested
    auto advance = [&](int t, int stage) {
        const int next = stage == NST - 1 ? 0 : stage + 1, after = next == NST - 1 ? 0 : next + 1;
        if (t + 1 < ntiles) store_stat(next, stat);
        publish(t + 1 < ntiles);
        if (t + 2 < ntiles) {
            stat = load_stat(t + 2);
            dma_tile(t + 2, after);
        }
    };
    // Two loops in sequence rather than one with two kinds of iteration: with two code paths through the
    // MFMAs in one loop the compiler merges their accumulator registers with copies at every iteration.
    int stage = 0, t = 0;
    const int ndiag = causal ? 2 : 0;
    for (; t < ndiag && t < ntiles; ++t, stage = stage == NST - 1 ? 0 : stage + 1) {  // the diagonal part
        advance(t, stage);
        const int q0 = qbeg + QT * t;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int qs = q0 + 32 * u;
            if (qs + 31 < kw0 || qs >= sh.s) continue;      // all its queries precede this wavefront's keys, or are past the end
            unit(stage, u, qs, std::true_type{});
        }
    }
    for (; t < ntiles; ++t, stage = stage == NST - 1 ? 0 : stage + 1) {               // fully visible tiles
        advance(t, stage);
        const int q0 = qbeg + QT * t;
        unit(stage, 0, q0, std::false_type{});
        unit(stage, 1, q0 + 32, std::false_type{});
    }
    if (kvalid) {
        E *orow = dqkv + ((size_t)b * sh.s + key) * pitch + (size_t)h * dh;
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                x4<E> ok, ov;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ok[i] = (E)(dk[c][4 * g + i] * scale);
                    ov[i] = (E)dv[c][4 * g + i];
                }
                if (c * 32 + 8 * g + 4 * half < dh) {
                    *reinterpret_cast<x4<E> *>(orow + d + c * 32 + 8 * g + 4 * half) = ok;
                    *reinterpret_cast<x4<E> *>(orow + 2 * d + c * 32 + 8 * g + 4 * half) = ov;
                }
            }
    }
}

// Explicit instantiations: the host compiler does not always emit the launch stub of a kernel template from its
// use in the launchers below alone.
#define LGA_INSTANTIATE_KERNELS(DH, OCC, E)                                                                          \
    template __global__ void attn_fwd_kernel<DH, E>(const E *, E *, float *, AttnShape);                             \
    template __global__ void attn_bwd_dq_kernel<DH, OCC, E>(const E *, const float *, const float *, const E *, E *, \
                                                            AttnShape);                                              \
    template __global__ void attn_bwd_dkv_kernel<DH, E>(const E *, const float *, const float *, const E *, E *,     \
                                                        AttnShape)
#define LGA_INSTANTIATE_TYPE(E)                                                                            \
    template __global__ void attn_delta_kernel<E>(const E *, const E *, float *, AttnShape, int);          \
    LGA_INSTANTIATE_KERNELS(32, 2, E);                                                                     \
    LGA_INSTANTIATE_KERNELS(64, 2, E);                                                                     \
    LGA_INSTANTIATE_KERNELS(96, 2, E);                                                                     \
    LGA_INSTANTIATE_KERNELS(128, 2, E);                                                                    \
    LGA_INSTANTIATE_KERNELS(160, 1, E)
LGA_INSTANTIATE_TYPE(bf16);
LGA_INSTANTIATE_TYPE(f16);
#undef LGA_INSTANTIATE_TYPE
#undef LGA_INSTANTIATE_KERNELS

// Dynamic LDS of the three kernels, in bytes.
// forward: three stages of a 64-key K tile and V tile
template <int DH> constexpr int smem_fwd() {
    return 3 * (TileDma<64, DH, pitch_rd<DH>()>::ELEMS + TileDma<64, DH, pitch_tr<DH>()>::ELEMS) * 2;
}
// dQ: two stages of a 64-key K tile and V tile
template <int DH> constexpr int smem_dq() {
    return 2 * (TileDma<64, DH, pitch_both<DH>()>::ELEMS + TileDma<64, DH, pitch_rd<DH>()>::ELEMS) * 2;
}
// dK/dV: three stages of a Q tile, a dO tile and the row statistics
template <int DH> constexpr int smem_dkv() { return 3 * (2 * 64 * DH * 2 + 2 * 64 * 4); }
template <int DH> constexpr int occ_dq() { return DH <= 128 ? 2 : 1; }     // workgroups per CU the dQ kernel's register budget is set for

// All three kernels use more dynamic LDS than a launch may ask for by default: raise the limit of every
// instantiation.  Called once, outside any launch path (see attn_prepare_kernels).
template <int DH, class E> hipError_t raise_lds_limits() {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(attn_fwd_kernel<DH, E>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem_fwd<DH>());
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(attn_bwd_dq_kernel<DH, occ_dq<DH>(), E>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem_dq<DH>());
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(attn_bwd_dkv_kernel<DH, E>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem_dkv<DH>());
    return e;
}
template <class E> hipError_t raise_lds_limits_all() {
    hipError_t e = raise_lds_limits<32, E>();
    if (e == hipSuccess) e = raise_lds_limits<64, E>();
    if (e == hipSuccess) e = raise_lds_limits<96, E>();
    if (e == hipSuccess) e = raise_lds_limits<128, E>();
    if (e == hipSuccess) e = raise_lds_limits<160, E>();
    return e;
}

template <int DH, class E> void fwd_dh(const E *qkv, E *out, float *lse, AttnShape sh, hipStream_t s) {
    dim3 grid((unsigned)(sh.n_seq * sh.heads) * ((sh.s + 255) / 256));
    char name[64];
    snprintf(name, sizeof(name), "attn_fwd_kernel<%d>", DH);
    const double pairs = (double)sh.n_seq * sh.heads * sh.s * sh.s * (sh.causal ? 0.5 : 1.0);      // visible (query, key) pairs
    const double act = (double)sh.n_seq * sh.s * sh.heads * sh.dh * 2.0;      // bytes of one [tokens, d] bf16 tensor
    ProfScope scope(name, 4.0 * pairs * sh.dh, 4.0 * act, s);
    hipLaunchKernelGGL((attn_fwd_kernel<DH, E>), grid, dim3(256), smem_fwd<DH>(), s, qkv, out, lse, sh);
}
template <int DH, class E>
void bwd_dh(const E *qkv, const float *lse, const float *delta, const E *dout, E *dqkv, AttnShape sh,
            hipStream_t s) {
    dim3 grid((unsigned)(sh.n_seq * sh.heads) * ((sh.s + 127) / 128));
    char name[64];
    const double pairs = (double)sh.n_seq * sh.heads * sh.s * sh.s * (sh.causal ? 0.5 : 1.0);
    const double act = (double)sh.n_seq * sh.s * sh.heads * sh.dh * 2.0;
    {
        snprintf(name, sizeof(name), "attn_bwd_dq_kernel<%d>", DH);
        ProfScope scope(name, 6.0 * pairs * sh.dh, 5.0 * act, s);
        hipLaunchKernelGGL((attn_bwd_dq_kernel<DH, occ_dq<DH>(), E>), grid, dim3(256), smem_dq<DH>(), s, qkv, lse, delta, dout,
                           dqkv, sh);
    }
    {
        snprintf(name, sizeof(name), "attn_bwd_dkv_kernel<%d>", DH);
        ProfScope scope(name, 8.0 * pairs * sh.dh, 6.0 * act, s);
        hipLaunchKernelGGL((attn_bwd_dkv_kernel<DH, E>), grid, dim3(256), smem_dkv<DH>(), s, qkv, lse, delta, dout, dqkv, sh);
    }
}

}  // namespace

// Head sizes 32, 64, 96, 128, 160 have kernels; any other multiple of 8 up to 160 runs in the next larger one with
// its extra columns read as zeros and not written.
bool attn_bf16_supports(int dh) { return dh >= 8 && dh <= 160 && dh % 8 == 0; }
static int padded_dh(int dh) { return (dh + 31) / 32 * 32; }

hipError_t attn_prepare_kernels() {
    hipError_t e = raise_lds_limits_all<bf16>();
    if (e == hipSuccess) e = raise_lds_limits_all<f16>();
    return e;
}

template <class E> void launch_attn_fwd_mfma(const E *qkv, E *out, float *lse, AttnShape sh, hipStream_t s) {
    if (sh.n_seq == 0 || sh.s == 0) return;
    if (!attn_bf16_supports(sh.dh)) {
        launch_attn_fwd_simple<E>(qkv, out, lse, sh, s);
        return;
    }
    (void)prepare_kernels();
    switch (padded_dh(sh.dh)) {
        case 32: fwd_dh<32, E>(qkv, out, lse, sh, s); break;
        case 64: fwd_dh<64, E>(qkv, out, lse, sh, s); break;
        case 96: fwd_dh<96, E>(qkv, out, lse, sh, s); break;
        case 128: fwd_dh<128, E>(qkv, out, lse, sh, s); break;
        case 160: fwd_dh<160, E>(qkv, out, lse, sh, s); break;
    }
}

template <class E>
void launch_attn_bwd_mfma(const E *qkv, const E *out, const float *lse, const E *dout, E *dqkv,
                          float *delta, AttnShape sh, hipStream_t s) {
    if (sh.n_seq == 0 || sh.s == 0) return;
    if (!attn_bf16_supports(sh.dh)) {
        launch_attn_bwd_simple<E>(qkv, out, lse, dout, dqkv, delta, sh, s);
        return;
    }
    (void)prepare_kernels();
    const size_t items = (size_t)sh.n_seq * sh.s * sh.heads;
    {
        ProfScope scope("attn_delta_kernel", 2.0 * items * sh.dh, 4.0 * items * sh.dh, s);
        const int items_per_block = 256 / (sh.dh / 8);                  // dh is a multiple of 8, at most 160
        hipLaunchKernelGGL(attn_delta_kernel<E>, dim3((unsigned)((items + items_per_block - 1) / items_per_block)), dim3(256), 0,
                           s, out, dout, delta, sh, items_per_block);
    }
    switch (padded_dh(sh.dh)) {
        case 32: bwd_dh<32, E>(qkv, lse, delta, dout, dqkv, sh, s); break;
        case 64: bwd_dh<64, E>(qkv, lse, delta, dout, dqkv, sh, s); break;
        case 96: bwd_dh<96, E>(qkv, lse, delta, dout, dqkv, sh, s); break;
        case 128: bwd_dh<128, E>(qkv, lse, delta, dout, dqkv, sh, s); break;
        case 160: bwd_dh<160, E>(qkv, lse, delta, dout, dqkv, sh, s); break;
    }
}

#define LGA_INSTANTIATE_ATTN(E)                                                                          \
    template void launch_attn_fwd_mfma<E>(const E *, E *, float *, AttnShape, hipStream_t);               \
    template void launch_attn_bwd_mfma<E>(const E *, const E *, const float *, const E *, E *, float *, \
                                          AttnShape, hipStream_t)
LGA_INSTANTIATE_ATTN(bf16);
LGA_INSTANTIATE_ATTN(f16);
#undef LGA_INSTANTIATE_ATTN

}  // namespace lga
