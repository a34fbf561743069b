// Softmax attention (causal or unmasked), correctness-mode kernels: one wavefront per (sequence, head, position).
// Scores, softmax and all sums in fp32; T is the storage type.  Used by the fp32 mode; the
// The 16-bit modes run the MFMA kernels in attention_bf16.hip.
#include "kernels.h"

namespace lga {

namespace {

// qkv row of token t: [Q(d) | K(d) | V(d)], head h at column h*dh inside each.
template <class T>
__global__ __launch_bounds__(64) void attn_fwd_simple_kernel(const T *__restrict__ qkv, T *__restrict__ out,
                                                             float *__restrict__ lse, AttnShape sh) {
    extern __shared__ float smem[];
    float *qs = smem;            // [dh]
    float *ps = smem + sh.dh;    // [s]
    const int lane = threadIdx.x;
    const int i = blockIdx.x % sh.s;
    const int h = (blockIdx.x / sh.s) % sh.heads;
    const int b = blockIdx.x / (sh.s * sh.heads);
    const int d = sh.heads * sh.dh;
    const size_t row3 = 3 * (size_t)d;
    const T *base = qkv + (size_t)b * sh.s * row3 + (size_t)h * sh.dh;
    const float scale = rsqrtf((float)sh.dh);
    for (int c = lane; c < sh.dh; c += 64) qs[c] = to_f32(base[(size_t)i * row3 + c]);
    __syncthreads();
    const int jend = sh.causal ? i + 1 : sh.s;      // keys [0, jend) are visible
    float mx = -INFINITY;
    for (int j = lane; j < jend; j += 64) {
        const T *kr = base + (size_t)j * row3 + d;
        float acc = 0.f;
        for (int c = 0; c < sh.dh; ++c) acc = fmaf(qs[c], to_f32(kr[c]), acc);
        acc *= scale;
        ps[j] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = lane; j < jend; j += 64) {
        const float e = expf(ps[j] - mx);
        ps[j] = e;
        sum += e;
    }
    sum = wave_sum(sum);
    __syncthreads();
    const float inv = 1.0f / sum;
    for (int c = lane; c < sh.dh; c += 64) {
        float acc = 0.f;
        for (int j = 0; j < jend; ++j) acc = fmaf(ps[j], to_f32(base[(size_t)j * row3 + 2 * d + c]), acc);
        out[((size_t)b * sh.s + i) * d + (size_t)h * sh.dh + c] = from_f32<T>(acc * inv);
    }
    if (lane == 0) lse[((size_t)b * sh.heads + h) * sh.s + i] = mx + logf(sum);
}

// (causal case written out) delta_i = sum_c dO_i[c] O_i[c];  dQ_i = scale * sum_{j<=i} dS_ij K_j,  dS_ij = P_ij (dO_i.V_j - delta_i)
template <class T>
__global__ __launch_bounds__(64) void attn_bwd_dq_simple_kernel(const T *__restrict__ qkv, const T *__restrict__ out,
                                                                const float *__restrict__ lse,
                                                                const T *__restrict__ dout, T *__restrict__ dqkv,
                                                                float *__restrict__ delta, AttnShape sh) {
    extern __shared__ float smem[];
    float *qs = smem;                 // [dh]
    float *dos = smem + sh.dh;        // [dh]
    float *ds = smem + 2 * sh.dh;     // [s]
    const int lane = threadIdx.x;
    const int i = blockIdx.x % sh.s;
    const int h = (blockIdx.x / sh.s) % sh.heads;
    const int b = blockIdx.x / (sh.s * sh.heads);
    const int d = sh.heads * sh.dh;
    const size_t row3 = 3 * (size_t)d;
    const T *base = qkv + (size_t)b * sh.s * row3 + (size_t)h * sh.dh;
    const size_t orow = ((size_t)b * sh.s + i) * d + (size_t)h * sh.dh;
    const float scale = rsqrtf((float)sh.dh);
    float dl = 0.f;
    for (int c = lane; c < sh.dh; c += 64) {
        qs[c] = to_f32(base[(size_t)i * row3 + c]);
        const float g = to_f32(dout[orow + c]);
        dos[c] = g;
        dl += g * to_f32(out[orow + c]);
    }
    dl = wave_sum(dl);
    const size_t stat = ((size_t)b * sh.heads + h) * sh.s + i;
    if (lane == 0) delta[stat] = dl;
    const float l = lse[stat];
    __syncthreads();
    const int jend = sh.causal ? i + 1 : sh.s;
    for (int j = lane; j < jend; j += 64) {
        const T *kr = base + (size_t)j * row3 + d;
        const T *vr = base + (size_t)j * row3 + 2 * d;
        float sc = 0.f, dp = 0.f;
        for (int c = 0; c < sh.dh; ++c) {
            sc = fmaf(qs[c], to_f32(kr[c]), sc);
            dp = fmaf(dos[c], to_f32(vr[c]), dp);
        }
        const float p = expf(sc * scale - l);
        ds[j] = p * (dp - dl);
    }
    __syncthreads();
    for (int c = lane; c < sh.dh; c += 64) {
        float acc = 0.f;
        for (int j = 0; j < jend; ++j) acc = fmaf(ds[j], to_f32(base[(size_t)j * row3 + d + c]), acc);
        dqkv[((size_t)b * sh.s + i) * row3 + (size_t)h * sh.dh + c] = from_f32<T>(acc * scale);
    }
}

// dV_j = sum_{i>=j} P_ij dO_i ;  dK_j = scale * sum_{i>=j} dS_ij Q_i
template <class T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_simple_kernel(const T *__restrict__ qkv,
                                                                 const float *__restrict__ lse,
                                                                 const T *__restrict__ dout, T *__restrict__ dqkv,
                                                                 const float *__restrict__ delta, AttnShape sh) {
    extern __shared__ float smem[];
    float *ks = smem;                   // [dh]
    float *vs = smem + sh.dh;           // [dh]
    float *ps = smem + 2 * sh.dh;       // [s]
    float *ds = ps + sh.s;              // [s]
    const int lane = threadIdx.x;
    const int j = blockIdx.x % sh.s;
    const int h = (blockIdx.x / sh.s) % sh.heads;
    const int b = blockIdx.x / (sh.s * sh.heads);
    const int d = sh.heads * sh.dh;
    const size_t row3 = 3 * (size_t)d;
    const T *base = qkv + (size_t)b * sh.s * row3 + (size_t)h * sh.dh;
    const T *dob = dout + (size_t)b * sh.s * d + (size_t)h * sh.dh;
    const float scale = rsqrtf((float)sh.dh);
    for (int c = lane; c < sh.dh; c += 64) {
        ks[c] = to_f32(base[(size_t)j * row3 + d + c]);
        vs[c] = to_f32(base[(size_t)j * row3 + 2 * d + c]);
    }
    __syncthreads();
    const size_t stat0 = ((size_t)b * sh.heads + h) * sh.s;
    const int ibeg = sh.causal ? j : 0;             // queries [ibeg, s) see key j
    for (int i = ibeg + lane; i < sh.s; i += 64) {
        const T *qr = base + (size_t)i * row3;
        const T *gr = dob + (size_t)i * d;
        float sc = 0.f, dp = 0.f;
        for (int c = 0; c < sh.dh; ++c) {
            sc = fmaf(to_f32(qr[c]), ks[c], sc);
            dp = fmaf(to_f32(gr[c]), vs[c], dp);
        }
        const float p = expf(sc * scale - lse[stat0 + i]);
        ps[i] = p;
        ds[i] = p * (dp - delta[stat0 + i]);
    }
    __syncthreads();
    for (int c = lane; c < sh.dh; c += 64) {
        float dv = 0.f, dk = 0.f;
        for (int i = ibeg; i < sh.s; ++i) {
            dv = fmaf(ps[i], to_f32(dob[(size_t)i * d + c]), dv);
            dk = fmaf(ds[i], to_f32(base[(size_t)i * row3 + c]), dk);
        }
        T *orow = dqkv + ((size_t)b * sh.s + j) * row3 + (size_t)h * sh.dh;
        orow[d + c] = from_f32<T>(dk * scale);
        orow[2 * d + c] = from_f32<T>(dv);
    }
}

}  // namespace

template <class T> void launch_attn_fwd_simple(const T *qkv, T *out, float *lse, AttnShape sh, hipStream_t s) {
    const size_t blocks = (size_t)sh.n_seq * sh.heads * sh.s;
    if (blocks == 0) return;
    const size_t smem = (size_t)(sh.dh + sh.s) * sizeof(float);
    ProfScope scope("attn_fwd_simple_kernel", 2.0 * blocks * sh.s * sh.dh, 4.0 * sizeof(T) * blocks * sh.dh, s);
    hipLaunchKernelGGL((attn_fwd_simple_kernel<T>), dim3((unsigned)blocks), dim3(64), smem, s, qkv, out, lse, sh);
}
template void launch_attn_fwd_simple<float>(const float *, float *, float *, AttnShape, hipStream_t);
template void launch_attn_fwd_simple<bf16>(const bf16 *, bf16 *, float *, AttnShape, hipStream_t);
template void launch_attn_fwd_simple<f16>(const f16 *, f16 *, float *, AttnShape, hipStream_t);

template <class T>
void launch_attn_bwd_simple(const T *qkv, const T *out, const float *lse, const T *dout, T *dqkv, float *delta,
                            AttnShape sh, hipStream_t s) {
    const size_t blocks = (size_t)sh.n_seq * sh.heads * sh.s;
    if (blocks == 0) return;
    const size_t smem_q = (size_t)(2 * sh.dh + sh.s) * sizeof(float);
    const size_t smem_kv = (size_t)(2 * sh.dh + 2 * sh.s) * sizeof(float);
    ProfScope scope("attn_bwd_simple_kernels", 7.0 * blocks * sh.s * sh.dh, 9.0 * sizeof(T) * blocks * sh.dh, s);
    hipLaunchKernelGGL((attn_bwd_dq_simple_kernel<T>), dim3((unsigned)blocks), dim3(64), smem_q, s, qkv, out, lse,
                       dout, dqkv, delta, sh);
    hipLaunchKernelGGL((attn_bwd_dkv_simple_kernel<T>), dim3((unsigned)blocks), dim3(64), smem_kv, s, qkv, lse, dout,
                       dqkv, delta, sh);
}
template void launch_attn_bwd_simple<float>(const float *, const float *, const float *, const float *, float *,
                                            float *, AttnShape, hipStream_t);
template void launch_attn_bwd_simple<bf16>(const bf16 *, const bf16 *, const float *, const bf16 *, bf16 *, float *,
                                           AttnShape, hipStream_t);
template void launch_attn_bwd_simple<f16>(const f16 *, const f16 *, const float *, const f16 *, f16 *, float *,
                                           AttnShape, hipStream_t);

}  // namespace lga
