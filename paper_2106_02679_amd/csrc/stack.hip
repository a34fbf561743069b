// C ABI and layer-major scheduler of the layered-gradient-accumulation layer-stack library.
// See include/lga.h for the contract of every entry point.
#include "../../include/lga.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include "kernels.h"

using namespace lga;

namespace {

thread_local std::string g_last_error;

int fail(int code, const std::string &msg) {
    g_last_error = msg;
    return code;
}

}  // namespace

namespace lga {
int set_last_error(int code, const char *msg) { return fail(code, msg); }
LaunchProfiler &profiler() {
    static LaunchProfiler p;
    return p;
}
hipError_t prepare_kernels() {
    static std::once_flag once;
    static hipError_t result = hipSuccess;
    std::call_once(once, [] {
        result = attn_prepare_kernels();
        if (result == hipSuccess) result = gemm_prepare_kernels();
    });
    return result;
}
}  // namespace lga

namespace {

#define LGA_HIP(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e_ = (expr);                                                                         \
        if (e_ != hipSuccess)                                                                           \
            return fail(e_ == hipErrorOutOfMemory ? LGA_ERR_OOM : LGA_ERR_HIP,                          \
                        std::string(#expr) + ": " + hipGetErrorString(e_));                             \
    } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Offsets (in elements) of one layer's tensors inside its flat canonical vector.
struct LayerLayout {
    size_t ln1_g, ln1_b, w_qkv, b_qkv, w_o, b_o, ln2_g, ln2_b, w_1, b_1, w_2, b_2, total, matrices;
};

LayerLayout make_layout(size_t d, size_t f) {
    LayerLayout o{};
    size_t p = 0;
    o.ln1_g = p; p += d;
    o.ln1_b = p; p += d;
    o.w_qkv = p; p += d * 3 * d;
    o.b_qkv = p; p += 3 * d;
    o.w_o = p; p += d * d;
    o.b_o = p; p += d;
    o.ln2_g = p; p += d;
    o.ln2_b = p; p += d;
    o.w_1 = p; p += d * f;
    o.b_1 = p; p += f;
    o.w_2 = p; p += f * d;
    o.b_2 = p; p += d;
    o.total = p;
    o.matrices = 4 * d * d + 2 * d * f;
    return o;
}

int validate_config(const lga_config *c) {
    if (!c) return fail(LGA_ERR_ARG, "config is NULL");
    if (c->dtype != LGA_FP32 && c->dtype != LGA_BF16 && c->dtype != LGA_FP16)
        return fail(LGA_ERR_ARG, "dtype must be LGA_FP32, LGA_BF16 or LGA_FP16");
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_ff < 1 || c->seq_len < 1 || c->micro_batch < 1 ||
        c->n_micro < 1)
        return fail(LGA_ERR_SHAPE, "every size must be >= 1");
    if (c->d_model % c->n_heads != 0) return fail(LGA_ERR_SHAPE, "d_model must be a multiple of n_heads");
    if (c->group < 1 || c->group > c->n_micro || c->n_micro % c->group != 0)
        return fail(LGA_ERR_SHAPE, "group must be in 1..n_micro and divide n_micro");
    if (c->wgrad_groups < 0 || c->wgrad_groups > c->n_micro / c->group)
        return fail(LGA_ERR_SHAPE, "wgrad_groups must be 0 (automatic) or in 1..n_micro/group");
    if (c->param_buffers < 0 || c->param_buffers > c->n_layers)
        return fail(LGA_ERR_SHAPE, "param_buffers must be 0 (one per layer) or in 1..n_layers");
    if (c->overlap < 0 || c->overlap > 3) return fail(LGA_ERR_ARG, "overlap must be a combination of LGA_OVERLAP_* bits");
    if (c->offload_checkpoints != 0 && c->offload_checkpoints != 1) return fail(LGA_ERR_ARG, "offload_checkpoints must be 0 or 1");
    if (c->attention != LGA_ATTN_CAUSAL && c->attention != LGA_ATTN_FULL)
        return fail(LGA_ERR_ARG, "attention must be LGA_ATTN_CAUSAL or LGA_ATTN_FULL");
    if (!(c->ln_eps >= 0.f)) return fail(LGA_ERR_ARG, "ln_eps must be >= 0");
    if (c->dtype == LGA_FP32 && (2.0 * c->seq_len + 2.0 * c->d_model / c->n_heads) * 4 > 60000)
        return fail(LGA_ERR_SHAPE, "fp32 mode: seq_len too long for the one-wavefront attention kernel's LDS rows");
    if (c->dtype != LGA_FP32) {
        const int dh = c->d_model / c->n_heads;
        if (dh % 8 != 0) return fail(LGA_ERR_SHAPE, "the 16-bit modes need head size d_h to be a multiple of 8");
        // head sizes without a fused attention kernel run the GEMM-built attention if seq_len is a multiple of 8
        // (at most 32768), else the one-wavefront kernels, like the fp32 mode
        if (!attn_bf16_supports(dh) && (c->seq_len % 8 != 0 || c->seq_len > 32768) && (2.0 * c->seq_len + 2.0 * dh) * 4 > 60000)
            return fail(LGA_ERR_SHAPE, "seq_len too long for the one-wavefront attention kernel's LDS rows (head size "
                                       "without an MFMA attention kernel)");
        if (c->d_model % 8 != 0 || c->d_ff % 8 != 0)
            return fail(LGA_ERR_SHAPE, "the 16-bit modes need d_model and d_ff to be multiples of 8");
        if (((long)c->group * c->micro_batch * c->seq_len) % 8 != 0)
            return fail(LGA_ERR_SHAPE, "the 16-bit modes need group * micro_batch * seq_len to be a multiple of 8");
    }
    // the 16-bit GEMMs address the 256 rows of an operand tile with 32-bit byte offsets inside a 1 GiB window, which
    // bounds every leading dimension: the widths, and the token count of one group (the weight-gradient GEMMs
    // contract over at least one group's tokens, stored with that pitch plus 64)
    if (c->dtype != LGA_FP32) {
        const long widest = std::max<long>(3L * c->d_model, c->d_ff + 64L);      // (d_ff-wide rows may be stored with a pitch of d_ff + 64)
        const long t_group = (long)c->group * c->micro_batch * c->seq_len;
        if (widest > kGemmMaxLd || t_group + 64 > kGemmMaxLd)
            return fail(LGA_ERR_SHAPE, "the 16-bit modes need 3 d_model, d_ff and group * micro_batch * seq_len + 64 to "
                                       "stay within 2 097 151 (leading dimensions of the GEMM operands)");
        if (c->wgrad_groups > 1 && (long)c->wgrad_groups * t_group + 64 > kGemmMaxLd)
            return fail(LGA_ERR_SHAPE, "wgrad_groups * group * micro_batch * seq_len + 64 must stay within 2 097 151 "
                                       "(row pitch of the merged weight-gradient GEMMs' operands); 0 chooses a count that does");
    }
    // kernels index rows and columns with int and elements with size_t
    const double tokens_group = (double)c->group * c->micro_batch * c->seq_len;
    if (tokens_group > 1.0e9 || 3.0 * c->d_model > 2.0e9 || (double)c->n_heads * c->micro_batch * c->group * ((c->seq_len + 127) / 128) > 2.0e9)
        return fail(LGA_ERR_SHAPE, "sizes overflow the index range");
    return LGA_OK;
}

// Arena plan: one allocation, every sub-buffer 256-byte aligned.
struct Plan {
    size_t w, m, v, grad, w16, w16t, ckpt, dact;
    size_t xT[4], dyT[4];      // transposed operands of the four weight-gradient GEMMs (16-bit modes)
    int wgrad_groups;          // groups whose tokens one weight-gradient GEMM contracts over
    size_t ldk;                // row pitch (elements) of the transposed operands
    size_t ldf;                // row pitch (elements) of the d_ff-wide activations u, gl, du
    size_t h, qkv, a, x1, h2, u, gl, du, dh2, dx1, da, dqkv, dh;
    size_t mean1, rstd1, mean2, rstd2, lse, delta, partial;
    size_t splitk, splitk_floats;   // partial results of weight-gradient GEMMs whose k range is split (narrow layers)
    size_t nonfinite;          // int per layer: the last checked Adam step found a non-finite gradient value
    size_t attn_ws, attn_ws_bytes;  // workspace of the GEMM-built attention (head sizes without a fused kernel)
    size_t total;
};

Plan make_plan(const lga_config &c) {
    Plan p{};
    const size_t d = c.d_model, f = c.d_ff, L = c.n_layers;
    const size_t P = make_layout(d, f).total;
    const bool is16 = c.dtype != LGA_FP32;
    const size_t esz = is16 ? 2 : 4;
    const size_t T = (size_t)c.n_micro * c.micro_batch * c.seq_len;
    const size_t t = (size_t)c.group * c.micro_batch * c.seq_len;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
    p.w = take(L * P * 4);
    p.m = take(L * P * 4);
    p.v = take(L * P * 4);
    p.grad = take((c.retain_grads ? L : (c.overlap & LGA_OVERLAP_ADAM) ? std::min<size_t>(2, L) : 1) * P * 4);
    const size_t nbuf = c.param_buffers ? (size_t)c.param_buffers : L;     // layers whose 16-bit copies are resident
    p.w16 = take(is16 ? nbuf * P * 2 : 0);
    p.w16t = take(is16 ? nbuf * P * 2 : 0);   // each matrix transposed, at its canonical offset
    p.ckpt = take((c.offload_checkpoints ? std::min<size_t>(2, L + 1) : L + 1) * T * d * esz);
    p.dact = take(T * d * esz);
    p.h = take(t * d * esz);
    p.qkv = take(t * 3 * d * esz);
    p.a = take(t * d * esz);
    p.x1 = take(t * d * esz);
    p.h2 = take(t * d * esz);
    // Rows of d_ff elements whose byte length is a multiple of 32 KB (d_ff = 49152: 96 KB) get a pitch 64 elements
    // longer: with the bare pitch the 256 rows of a GEMM operand tile start in few memory channels, and the two GEMMs
    // that contract over d_ff lose 7 % (1.50 against 1.61 PFLOP/s; 1 % of the step).  Measured without effect on rows
    // of 16 KB (d_ff = 8192), 6 KB and 200 KB, and on the d_model- and 3 d_model-wide rows of all configurations.
    p.ldf = (is16 && (f * esz) % 32768 == 0) ? f + 64 : f;
    p.u = take(t * p.ldf * esz);
    p.gl = take(t * p.ldf * esz);
    p.du = take(t * p.ldf * esz);
    p.dh2 = take(t * d * esz);
    p.dx1 = take(t * d * esz);
    p.da = take(t * d * esz);
    p.dqkv = take(t * 3 * d * esz);
    p.dh = take(t * d * esz);
    // Transposed operands of the weight-gradient GEMMs: [in][ldk] copies of their inputs and [out][ldk]
    // copies of their output gradients, wgrad_groups groups side by side along the token axis.  The pitch
    // is padded by 64 elements: the unpadded one is a large power of two, which maps every row of an
    // operand tile to the same memory channel.
    const size_t groups = (size_t)c.n_micro / c.group;
    const size_t rows = 2 * f + 8 * d;                      // in + out over the four matrices
    size_t wb = c.wgrad_groups ? (size_t)c.wgrad_groups : 1;
    if (is16 && c.wgrad_groups == 0) {
        // automatic: as many groups as keep these buffers within a quarter of everything else
        // ... and keep their row pitch within what the GEMM's loads can address
        wb = groups;
        while (wb > 1 && (rows * (wb * t + 64) * 2 > off / 4 || wb * t + 64 > (size_t)kGemmMaxLd)) --wb;
    }
    p.wgrad_groups = (int)wb;
    p.ldk = wb * t + 64;
    const int wg_in[4] = {(int)f, (int)d, (int)d, (int)d};          // W_2, W_1, W_o, W_qkv
    const int wg_out[4] = {(int)d, (int)f, (int)d, (int)(3 * d)};
    for (int i = 0; i < 4; ++i) {
        p.xT[i] = take(is16 ? (size_t)wg_in[i] * p.ldk * 2 : 0);
        p.dyT[i] = take(is16 ? (size_t)wg_out[i] * p.ldk * 2 : 0);
    }
    p.splitk_floats = 0;
    if (is16)
        for (int i = 0; i < 4; ++i) {
            const size_t slices = (size_t)gemm_splitk_slices(wg_in[i], wg_out[i], 0);
            if (slices > 1) p.splitk_floats = std::max(p.splitk_floats, slices * wg_in[i] * wg_out[i]);
        }
    p.splitk = take(p.splitk_floats * 4);
    p.mean1 = take(t * 4);
    p.rstd1 = take(t * 4);
    p.mean2 = take(t * 4);
    p.rstd2 = take(t * 4);
    const size_t stats = (size_t)c.group * c.micro_batch * c.n_heads * c.seq_len;
    p.lse = take(stats * 4);
    p.delta = take(stats * 4);
    const size_t widest = std::max<size_t>(3 * d, f);
    p.partial = take(std::max(colsum_partial_floats((int)t, (int)widest), layernorm_bwd_partial_floats((int)t, (int)c.d_model)) * 4);
    p.nonfinite = take(L * 4);          // one flag per layer, see lga_adam.skip_nonfinite
    // head sizes without a fused attention kernel: score matrices of as many heads of one sequence as fit 4 GiB
    p.attn_ws_bytes = 0;
    if (is16 && !attn_bf16_supports((int)(d / c.n_heads)) && c.seq_len % 8 == 0 && c.seq_len <= 32768) {
        const size_t per_head = attn_gemm_workspace_bytes(c.seq_len, 1);
        const size_t heads = std::min<size_t>(c.n_heads, std::max<size_t>(1, ((size_t)4 << 30) / per_head));
        p.attn_ws_bytes = heads * per_head;
    }
    p.attn_ws = take(p.attn_ws_bytes);
    p.total = off;
    return p;
}

}  // namespace

struct lga_stack {
    lga_config cfg;
    LayerLayout lay;
    Plan plan;
    hipStream_t stream;
    char *arena;
    size_t P, T, t;          // params per layer, tokens per step, tokens per group
    // input_valid[l]: boundary l holds the input layer l's last forward saw, and the layer's weights have not
    // changed since - what the layer's backward (which recomputes from that input) needs
    std::vector<char> input_valid;
    bool have_forward() const {
        for (char ok : input_valid) if (!ok) return false;
        return true;
    }
    void set_forward(bool ok) { std::fill(input_valid.begin(), input_valid.end(), (char)ok); }
    std::vector<int> grad_owner;   // which layer's gradient each gradient buffer currently holds (-1: none)
    int ngrad;                     // gradient buffers: layer l uses buffer l % ngrad
    // overlap mode: Adam steps and restores run on a second stream beside the layer sweeps
    hipStream_t aux;
    hipEvent_t ev_fork;                        // "everything enqueued on the main stream so far"
    std::vector<hipEvent_t> ev_w16, ev_grad;   // last write of each 16-bit parameter buffer / last read of each gradient buffer on aux
    std::vector<char> w16_pending, grad_pending;   // the main stream has not waited for that event yet
    // checkpoint offload: all boundaries live in pinned host memory; the device keeps two slots, boundary b in slot b % 2
    char *host_ckpt;
    int dev_boundary[2];           // which boundary each device slot holds (-1: none)
    hipEvent_t ev_ck[2];           // last transfer (either direction) of each slot on aux
    char ck_pending[2];            // the main stream has not waited for that event yet
    int nbuf;                      // 16-bit parameter buffers: layer l uses buffer l % nbuf
    std::vector<int> w16_owner;    // which layer's 16-bit copies each of them currently holds (-1: none)
    uint64_t restores;             // casts of a layer's parameters into a buffer since creation

    template <class X> X *at(size_t off) const { return reinterpret_cast<X *>(arena + off); }
    float *w(int l) const { return at<float>(plan.w) + (size_t)l * P; }
    float *m(int l) const { return at<float>(plan.m) + (size_t)l * P; }
    float *v(int l) const { return at<float>(plan.v) + (size_t)l * P; }
    // 16-bit parameter copies, in the configured 16-bit format (E = bf16 or f16; uint16_t where only bits move)
    template <class E = uint16_t> E *w16(int l) const { return at<E>(plan.w16) + (size_t)(l % nbuf) * P; }
    template <class E = uint16_t> E *w16t(int l) const { return at<E>(plan.w16t) + (size_t)(l % nbuf) * P; }
    bool is16() const { return cfg.dtype != LGA_FP32; }
    int *nonfinite(int l) const { return at<int>(plan.nonfinite) + l; }
    bool w16_resident(int l) const { return w16_owner[l % nbuf] == l; }
    int grad_slot(int l) const { return l % ngrad; }
    float *grad(int l) const { return at<float>(plan.grad) + (size_t)grad_slot(l) * P; }
    size_t esz() const { return is16() ? 2 : 4; }
    size_t boundary_bytes() const { return T * cfg.d_model * esz(); }
    // device address of a boundary activation (offload mode: of the slot it lives in while it is on the device)
    char *ckpt(int boundary) const {
        return arena + plan.ckpt + (size_t)(cfg.offload_checkpoints ? boundary % 2 : boundary) * boundary_bytes();
    }
    char *host_boundary(int boundary) const { return host_ckpt + (size_t)boundary * boundary_bytes(); }
};

namespace {

// Set when a GEMM launcher refused its arguments (validate_config rules that out); finish() turns it into an error.
bool g_gemm_refused = false;

template <class T> void gemm(const GemmParams<T> &p, bool akm, bool bkm, Epilogue e, hipStream_t s) {
    if constexpr (std::is_same<T, float>::value) launch_gemm_f32(p, akm, bkm, e, s);
    else if (!launch_gemm_mfma<T>(p, akm, bkm, e, s)) g_gemm_refused = true;
}

// The weights the GEMMs read: fp32 masters in fp32 mode, the 16-bit copy in the 16-bit modes.
template <class T> const T *gemm_weights(const lga_stack *st, int l) {
    if constexpr (std::is_same<T, float>::value) return st->w(l);
    else return st->w16<T>(l);
}

// Refresh layer l's transposed 16-bit matrices ([out][in]) from its 16-bit copy ([in][out]): the
// forward GEMMs read them so that both of their operands are k-contiguous.
void refresh_transposed_weights(lga_stack *st, int l, hipStream_t s) {
    const int d = st->cfg.d_model, f = st->cfg.d_ff;
    const LayerLayout &o = st->lay;
    const uint16_t *w = st->w16(l);
    uint16_t *wt = st->w16t(l);
    launch_transpose16(w + o.w_qkv, wt + o.w_qkv, d, 3 * d, 3 * d, d, s);
    launch_transpose16(w + o.w_o, wt + o.w_o, d, d, d, d, s);
    launch_transpose16(w + o.w_1, wt + o.w_1, d, f, f, d, s);
    launch_transpose16(w + o.w_2, wt + o.w_2, f, d, d, f, s);
}

// ---- overlap mode plumbing -----------------------------------------------------------------------
// Work given to the second stream starts after everything enqueued on the main stream so far.
void fork_aux(lga_stack *st) {
    (void)hipEventRecord(st->ev_fork, st->stream);
    (void)hipStreamWaitEvent(st->aux, st->ev_fork, 0);
}
// The main stream waits for the second stream's last write of a 16-bit parameter buffer / last read of a
// gradient buffer, if it has not done so yet.
void wait_w16(lga_stack *st, int slot) {
    if (!st->w16_pending[slot]) return;
    (void)hipStreamWaitEvent(st->stream, st->ev_w16[slot], 0);
    st->w16_pending[slot] = 0;
}
void wait_grad(lga_stack *st, int slot) {
    if (!st->grad_pending[slot]) return;
    (void)hipStreamWaitEvent(st->stream, st->ev_grad[slot], 0);
    st->grad_pending[slot] = 0;
}
void join_aux(lga_stack *st) {
    for (size_t i = 0; i < st->w16_pending.size(); ++i) wait_w16(st, (int)i);
    for (size_t i = 0; i < st->grad_pending.size(); ++i) wait_grad(st, (int)i);
}
// ---- checkpoint offload (appendix C.5, "CPU-GPU transfers") ------------------------------------------------
// Transfers run on the second stream, ordered against the main stream by one event per device slot.
void wait_slot(lga_stack *st, int slot) {
    if (!st->ck_pending[slot]) return;
    (void)hipStreamWaitEvent(st->stream, st->ev_ck[slot], 0);
    st->ck_pending[slot] = 0;
}
// Boundary b, complete on the device once everything enqueued on the main stream so far has run, goes to the host.
void save_boundary(lga_stack *st, int b) {
    fork_aux(st);
    (void)hipMemcpyAsync(st->host_boundary(b), st->ckpt(b), st->boundary_bytes(), hipMemcpyDeviceToHost, st->aux);
    (void)hipEventRecord(st->ev_ck[b % 2], st->aux);
    st->ck_pending[b % 2] = 1;
}
// Boundary b comes back into its slot, whose present content nothing enqueued after this call uses any more.  The
// copy starts when the main stream reaches this point and runs beside what is enqueued next.
void fetch_boundary(lga_stack *st, int b) {
    if (st->dev_boundary[b % 2] == b) return;
    fork_aux(st);
    if (st->ck_pending[b % 2]) (void)hipStreamWaitEvent(st->aux, st->ev_ck[b % 2], 0);   // same stream: ordered anyway
    (void)hipMemcpyAsync(st->ckpt(b), st->host_boundary(b), st->boundary_bytes(), hipMemcpyHostToDevice, st->aux);
    (void)hipEventRecord(st->ev_ck[b % 2], st->aux);
    st->ck_pending[b % 2] = 1;
    st->dev_boundary[b % 2] = b;
}
// The main stream is about to overwrite boundary b's slot with that boundary: the slot's last transfer must be over.
void claim_slot(lga_stack *st, int b) {
    wait_slot(st, b % 2);
    st->dev_boundary[b % 2] = b;
}
void join_offload(lga_stack *st) {
    wait_slot(st, 0);
    wait_slot(st, 1);
}

void release_stack(lga_stack *st) {
    if (st->aux) (void)hipStreamSynchronize(st->aux);
    for (hipEvent_t ev : st->ev_w16) if (ev) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : st->ev_grad) if (ev) (void)hipEventDestroy(ev);
    if (st->ev_fork) (void)hipEventDestroy(st->ev_fork);
    for (hipEvent_t ev : st->ev_ck) if (ev) (void)hipEventDestroy(ev);
    if (st->aux) (void)hipStreamDestroy(st->aux);
    if (st->host_ckpt) (void)hipHostFree(st->host_ckpt);
    if (st->arena) (void)hipFree(st->arena);
    delete st;
}

// "Restore" of the paper's figure 2 and table C.1: make the 16-bit copies of layer l's parameters available
// before the layer is used.  With one buffer per layer they always are (every Adam step rewrites them); with
// fewer (param_buffers), the layer's fp32 masters are cast into its buffer whenever another layer has used it
// in the meantime - once per layer and pass in the layered order, once per layer, pass AND micro-batch in the
// micro-batch-major order.
void restore_weights(lga_stack *st, int l) {
    const int slot = l % st->nbuf;
    hipStream_t s = st->stream;
    if (st->cfg.overlap) {
        fork_aux(st);               // the buffer's previous layer is no longer read by anything enqueued after this
        s = st->aux;
    }
    if (st->cfg.dtype == LGA_FP16) launch_cast_f32_to_16<f16>(st->w(l), st->w16<f16>(l), st->P, s);
    else launch_cast_f32_to_16<bf16>(st->w(l), st->w16<bf16>(l), st->P, s);
    st->w16_owner[slot] = l;
    refresh_transposed_weights(st, l, s);
    if (st->cfg.overlap) {
        (void)hipEventRecord(st->ev_w16[slot], st->aux);
        st->w16_pending[slot] = 1;
    }
    ++st->restores;
}
void ensure_weights(lga_stack *st, int l) {
    if (!st->is16()) return;
    if (!st->w16_resident(l)) restore_weights(st, l);
    if (st->cfg.overlap) wait_w16(st, l % st->nbuf);
}
// Overlap mode: start restoring layer `next` while layer `cur`'s sweep, enqueued after this call, runs.
void prefetch_weights(lga_stack *st, int next, int cur) {
    if (!st->is16() || !st->cfg.overlap || next < 0 || next >= st->cfg.n_layers) return;
    if (st->w16_resident(next) || next % st->nbuf == cur % st->nbuf) return;
    restore_weights(st, next);
}

// Forward of layer l on one micro-batch group (paper section 5 "Model"; pre-LN residual form).
// x_in: [t, d] group slice of the layer's input checkpoint.  y_out: group slice of the next
// checkpoint, or NULL when this is the backward pass's recompute (the second feed-forward GEMM's
// output is not needed there, so it is not recomputed).
template <class T> void layer_forward(lga_stack *st, int l, const T *x_in, T *y_out) {
    const lga_config &c = st->cfg;
    const int d = c.d_model, f = c.d_ff, t = (int)st->t;
    const LayerLayout &o = st->lay;
    const float *pf = st->w(l);
    const T *pw = gemm_weights<T>(st, l);
    hipStream_t s = st->stream;
    T *h = st->at<T>(st->plan.h), *qkv = st->at<T>(st->plan.qkv), *a = st->at<T>(st->plan.a);
    T *x1 = st->at<T>(st->plan.x1), *h2 = st->at<T>(st->plan.h2), *u = st->at<T>(st->plan.u);
    T *gl = st->at<T>(st->plan.gl);
    float *lse = st->at<float>(st->plan.lse);
    const AttnShape ash{c.group * c.micro_batch, c.seq_len, c.n_heads, d / c.n_heads, c.attention == LGA_ATTN_CAUSAL};

    // y[t, out] = x[t, in] W[in, out]: fp32 mode reads W as stored; the 16-bit modes read the transposed copy
    // W^T[out, in], so both operands are k-contiguous.
    constexpr bool k16bit = !std::is_same<T, float>::value;
    const T *pwt = pw;
    if constexpr (k16bit) pwt = st->w16t<T>(l);
    const int ldf = (int)st->plan.ldf;                       // pitch of u and gl
    auto fwd_gemm = [&](GemmParams<T> g, size_t w_off, int in, int out, Epilogue e, int lda = 0, int ldc = 0) {
        g.M = t; g.N = out; g.K = in; g.lda = lda ? lda : in; g.ldc = ldc ? ldc : out;
        g.B = pwt + w_off;
        g.ldb = k16bit ? in : out;
        gemm<T>(g, true, k16bit, e, s);
    };

    launch_layernorm_fwd<T>(x_in, pf + o.ln1_g, pf + o.ln1_b, h, st->at<float>(st->plan.mean1),
                            st->at<float>(st->plan.rstd1), t, d, c.ln_eps, s);
    GemmParams<T> g{};
    g.A = h; g.out = qkv; g.bias = pf + o.b_qkv;
    fwd_gemm(g, o.w_qkv, d, 3 * d, EPI_BIAS);
    if constexpr (std::is_same<T, float>::value) launch_attn_fwd_simple<float>(qkv, a, lse, ash, s);
    else if (!attn_bf16_supports(ash.dh) && attn_gemm_supports(ash, st->plan.attn_ws_bytes))
        launch_attn_fwd_gemm<T>(qkv, a, lse, ash, st->arena + st->plan.attn_ws, st->plan.attn_ws_bytes, s);
    else launch_attn_fwd_mfma<T>(qkv, a, lse, ash, s);
    g = GemmParams<T>{};
    g.A = a; g.out = x1; g.bias = pf + o.b_o; g.aux = x_in;
    fwd_gemm(g, o.w_o, d, d, EPI_BIAS_RESID);
    launch_layernorm_fwd<T>(x1, pf + o.ln2_g, pf + o.ln2_b, h2, st->at<float>(st->plan.mean2),
                            st->at<float>(st->plan.rstd2), t, d, c.ln_eps, s);
    g = GemmParams<T>{};
    g.A = h2; g.out = gl; g.out2 = u; g.bias = pf + o.b_1;
    fwd_gemm(g, o.w_1, d, f, EPI_BIAS_GELU, 0, ldf);
    if (y_out) {
        g = GemmParams<T>{};
        g.A = gl; g.out = y_out; g.bias = pf + o.b_2; g.aux = x1;
        fwd_gemm(g, o.w_2, f, d, EPI_BIAS_RESID, ldf, 0);
    }
}

// How one group's weight gradients enter the layer's fp32 gradient buffer.
struct GradStep {
    float beta;       // vectors (biases, LayerNorm): 0 for the layer's first group, then 1
    float beta_mat;   // matrices: 0 for the first weight-gradient GEMM of the layer, then 1
    int slot;         // 16-bit modes: position of this group's tokens in the transposed operand buffers
    bool flush;       // 16-bit modes: run the matrix GEMMs now, over slots 0..slot
};

// Backward of layer l on one group whose intermediates were just recomputed by layer_forward.
// dy: [t, d] group slice of the running activation gradient, overwritten with dx.
// gbuf: the layer's fp32 gradient buffer (canonical layout).
//
// The 16-bit modes merge the weight-gradient GEMMs of consecutive groups of a layer (possible because the
// layered order visits all micro-batches of a layer back to back): each group only appends its
// transposed operands, and one GEMM then contracts over all their tokens.  The accumulation over
// micro-batches that the fp32 buffer would do by read-modify-write happens inside the GEMM's
// k loop instead, so the buffer is touched once per merged GEMM rather than once per group.
template <class T> void layer_backward(lga_stack *st, int l, const T *x_in, T *dy, float *gbuf, GradStep gs) {
    const float beta = gs.beta;
    const lga_config &c = st->cfg;
    const int d = c.d_model, f = c.d_ff, t = (int)st->t;
    const LayerLayout &o = st->lay;
    const float *pf = st->w(l);
    const T *pw = gemm_weights<T>(st, l);
    hipStream_t s = st->stream;
    T *h = st->at<T>(st->plan.h), *qkv = st->at<T>(st->plan.qkv), *a = st->at<T>(st->plan.a);
    T *x1 = st->at<T>(st->plan.x1), *h2 = st->at<T>(st->plan.h2), *u = st->at<T>(st->plan.u);
    T *gl = st->at<T>(st->plan.gl), *du = st->at<T>(st->plan.du), *dh2 = st->at<T>(st->plan.dh2);
    T *dx1 = st->at<T>(st->plan.dx1), *da = st->at<T>(st->plan.da), *dqkv = st->at<T>(st->plan.dqkv);
    T *dh = st->at<T>(st->plan.dh);
    float *mean1 = st->at<float>(st->plan.mean1), *rstd1 = st->at<float>(st->plan.rstd1);
    float *mean2 = st->at<float>(st->plan.mean2), *rstd2 = st->at<float>(st->plan.rstd2);
    float *lse = st->at<float>(st->plan.lse), *delta = st->at<float>(st->plan.delta);
    float *partial = st->at<float>(st->plan.partial);
    const AttnShape ash{c.group * c.micro_batch, c.seq_len, c.n_heads, d / c.n_heads, c.attention == LGA_ATTN_CAUSAL};

    // gW[in, out] (+)= X[t, in]^T dY[t, out], contracted over tokens.  The 16-bit modes first write X^T [in][.]
    // and dY^T [out][.] (two HBM-bound passes, ~1 % of the GEMM's time) so that the GEMM reads both
    // operands k-contiguous; `which` names the matrix's pair of transposed buffers.
    const int ldf = (int)st->plan.ldf;                       // pitch of u, gl and du
    // ldx, ldy: row pitches of X and dY where they differ from the widths
    auto wgrad = [&](int which, const T *X, int in, const T *dY, int out, size_t w_off, size_t b_off, int ldx = 0, int ldy = 0) {
        if (!ldx) ldx = in;
        if (!ldy) ldy = out;
        GemmParams<T> g{};
        g.M = in; g.N = out;
        g.outf = gbuf + w_off; g.ldc = out;
        if constexpr (std::is_same<T, float>::value) {
            g.K = t; g.beta = beta;
            g.A = X; g.lda = ldx; g.B = dY; g.ldb = ldy;
            gemm<T>(g, false, false, EPI_ACCUM_F32, s);
        } else {
            const int ldk = (int)st->plan.ldk;
            T *xT = st->at<T>(st->plan.xT[which]), *dyT = st->at<T>(st->plan.dyT[which]);
            launch_transpose16(X, xT + (size_t)gs.slot * t, t, in, ldx, ldk, s);
            // the bias gradient is the column sum of dY: taken from the tiles as they are transposed
            launch_transpose16_colsum<T>(dY, dyT + (size_t)gs.slot * t, t, out, ldy, ldk, beta, gbuf + b_off, partial, s);
            if (gs.flush) {
                g.K = (gs.slot + 1) * t; g.beta = gs.beta_mat;
                g.A = xT; g.lda = ldk; g.B = dyT; g.ldb = ldk;
                g.partial = st->at<float>(st->plan.splitk); g.partial_floats = st->plan.splitk_floats;
                gemm<T>(g, true, true, EPI_ACCUM_F32, s);
            }
        }
        if constexpr (std::is_same<T, float>::value)
            launch_colsum<T>(dY, nullptr, nullptr, nullptr, t, out, ldy, beta, gbuf + b_off, nullptr, partial, s);
    };
    // lda: row pitch of dY, ldc: of dX and aux, where they differ from the widths
    auto dgrad = [&](const T *dY, int out, size_t w_off, int in, T *dX, Epilogue e, const T *aux, int lda = 0, int ldc = 0) {
        GemmParams<T> g{};
        g.A = dY; g.lda = lda ? lda : out; g.B = pw + w_off; g.ldb = out; g.M = t; g.N = in; g.K = out;
        g.out = dX; g.ldc = ldc ? ldc : in; g.aux = aux;
        gemm<T>(g, true, true, e, s);
    };

    // y = x1 + gelu(u) W2 + b2
    wgrad(0, gl, f, dy, d, o.w_2, o.b_2, ldf, 0);
    dgrad(dy, d, o.w_2, f, du, EPI_MUL_DGELU, u, 0, ldf);    // du = (dy W2^T) * gelu'(u)
    // u = h2 W1 + b1
    wgrad(1, h2, d, du, f, o.w_1, o.b_1, 0, ldf);
    dgrad(du, f, o.w_1, d, dh2, EPI_STORE, nullptr, ldf, 0);
    // h2 = LN2(x1); dx1 = dy + LN2'(dh2)
    launch_layernorm_bwd_dx<T>(dh2, x1, mean2, rstd2, pf + o.ln2_g, dy, dx1, t, d, s, beta, gbuf + o.ln2_b, gbuf + o.ln2_g, partial);
    // x1 = x + a Wo + bo
    wgrad(2, a, d, dx1, d, o.w_o, o.b_o);
    dgrad(dx1, d, o.w_o, d, da, EPI_STORE, nullptr);
    if constexpr (std::is_same<T, float>::value) launch_attn_bwd_simple<float>(qkv, a, lse, da, dqkv, delta, ash, s);
    else if (!attn_bf16_supports(ash.dh) && attn_gemm_supports(ash, st->plan.attn_ws_bytes))
        launch_attn_bwd_gemm<T>(qkv, a, lse, da, dqkv, delta, ash, st->arena + st->plan.attn_ws, st->plan.attn_ws_bytes, s);
    else launch_attn_bwd_mfma<T>(qkv, a, lse, da, dqkv, delta, ash, s);
    // qkv = h Wqkv + bqkv
    wgrad(3, h, d, dqkv, 3 * d, o.w_qkv, o.b_qkv);
    dgrad(dqkv, 3 * d, o.w_qkv, d, dh, EPI_STORE, nullptr);
    // h = LN1(x); dx = dx1 + LN1'(dh)
    launch_layernorm_bwd_dx<T>(dh, x_in, mean1, rstd1, pf + o.ln1_g, dx1, dy, t, d, s, beta, gbuf + o.ln1_b, gbuf + o.ln1_g, partial);
}

// async: on the second stream, after everything enqueued so far (overlap mode, fused Adam of the layered order)
void adam_layer(lga_stack *st, int l, const lga_adam &hp, bool async = false) {
    hipStream_t s = st->stream;
    if (async) {
        fork_aux(st);
        s = st->aux;
    }
    // the 16-bit copies are rewritten only if the layer still owns its buffer; otherwise the next use restores them
    const bool copies = st->is16() && st->w16_resident(l);
    if (copies && !async && st->cfg.overlap) wait_w16(st, l % st->nbuf);
    // Gradient scaling (section 2.2): the caller multiplied the output gradient by loss_scale, so the accumulated
    // gradient is divided by it here; with skip_nonfinite the gradient is tested first and an update whose gradient
    // overflowed is left out as a whole (parameters, moments and 16-bit copies keep their values).
    const float grad_mul = (hp.loss_scale > 0.f && hp.loss_scale != 1.f) ? 1.0f / hp.loss_scale : 1.0f;
    int *flag = nullptr;
    if (hp.skip_nonfinite) {
        flag = st->nonfinite(l);
        launch_fill_const(reinterpret_cast<float *>(flag), 1, 0.f, s);        // all bits zero
        launch_nonfinite_flag(st->grad(l), st->P, flag, s);
    }
    if (st->cfg.dtype == LGA_FP16)
        launch_adam<f16>(st->w(l), st->m(l), st->v(l), st->grad(l), copies ? st->w16<f16>(l) : nullptr, st->P, hp.lr,
                         hp.beta1, hp.beta2, hp.eps, hp.step, grad_mul, flag, s);
    else
        launch_adam<bf16>(st->w(l), st->m(l), st->v(l), st->grad(l), copies ? st->w16<bf16>(l) : nullptr, st->P, hp.lr,
                          hp.beta1, hp.beta2, hp.eps, hp.step, grad_mul, flag, s);
    if (copies) refresh_transposed_weights(st, l, s);
    if (async) {
        (void)hipEventRecord(st->ev_grad[st->grad_slot(l)], st->aux);
        st->grad_pending[st->grad_slot(l)] = 1;
        if (copies) {
            (void)hipEventRecord(st->ev_w16[l % st->nbuf], st->aux);
            st->w16_pending[l % st->nbuf] = 1;
        }
    }
}

int check_adam(const lga_adam *a) {
    if (a->step < 1) return fail(LGA_ERR_STATE, "Adam step t must be >= 1");
    if (!(a->beta1 >= 0.f && a->beta1 < 1.f && a->beta2 >= 0.f && a->beta2 < 1.f))
        return fail(LGA_ERR_ARG, "Adam betas must lie in [0, 1)");
    if (!(a->loss_scale >= 0.f) || std::isinf(a->loss_scale)) return fail(LGA_ERR_ARG, "loss_scale must be finite and >= 0");
    if (a->skip_nonfinite != 0 && a->skip_nonfinite != 1) return fail(LGA_ERR_ARG, "skip_nonfinite must be 0 or 1");
    return LGA_OK;
}

int finish(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(LGA_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
    if (g_gemm_refused) {
        g_gemm_refused = false;
        return fail(LGA_ERR_SHAPE, std::string(what) + ": a GEMM launch was refused (operand layout or leading dimension)");
    }
    return LGA_OK;
}

// The sweeps enqueue thousands of launches and copies, set function attributes on first use and (with a second
// stream or offload) record and wait for events; none of that has been shown to work on a stream that is being
// captured into a HIP graph, so such a stream is refused before anything is enqueued.
int refuse_capture(const lga_stack *st, const char *what) {
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    const hipError_t e = hipStreamIsCapturing(st->stream, &status);
    if (e != hipSuccess) (void)hipGetLastError();       // the legacy stream cannot even be asked while another stream captures
    if (e != hipSuccess || status != hipStreamCaptureStatusNone)
        return fail(LGA_ERR_STATE, std::string(what) + ": the stack's stream is being captured into a graph (or cannot be "
                                   "used while another stream is): graph capture of the layer sweeps is not supported");
    return LGA_OK;
}

template <class T> int forward_layered_t(lga_stack *st, const void *x, void *y) {
    const lga_config &c = st->cfg;
    const size_t act_bytes = st->T * c.d_model * sizeof(T);
    const bool offload = c.offload_checkpoints != 0;
    if (offload) claim_slot(st, 0);
    LGA_HIP(hipMemcpyAsync(st->ckpt(0), x, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    if (offload) save_boundary(st, 0);
    const int groups = c.n_micro / c.group;
    const size_t gstride = st->t * c.d_model;
    for (int l = 0; l < c.n_layers; ++l) {                 // layers outside ...
        // offload mode: boundary l + 1 takes the slot of boundary l - 1, which is on its way to the host since the
        // end of layer l - 2's sweep; its own copy to the host then runs beside layer l + 1's sweep
        if (offload) claim_slot(st, l + 1);
        const T *in = reinterpret_cast<const T *>(st->ckpt(l));
        T *out = reinterpret_cast<T *>(st->ckpt(l + 1));
        ensure_weights(st, l);
        prefetch_weights(st, l + 1, l);
        for (int gi = 0; gi < groups; ++gi)                 // ... micro-batches inside
            layer_forward<T>(st, l, in + gi * gstride, out + gi * gstride);
        if (offload) save_boundary(st, l + 1);
    }
    if (y) LGA_HIP(hipMemcpyAsync(y, st->ckpt(c.n_layers), act_bytes, hipMemcpyDeviceToDevice, st->stream));
    if (offload) join_offload(st);
    return finish("lga_forward_layered");
}

template <class T> int backward_layered_t(lga_stack *st, const void *dy, void *dx, const lga_adam *fused) {
    const lga_config &c = st->cfg;
    const size_t act_bytes = st->T * c.d_model * sizeof(T);
    T *dact = st->at<T>(st->plan.dact);
    LGA_HIP(hipMemcpyAsync(dact, dy, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    const int groups = c.n_micro / c.group;
    const size_t gstride = st->t * c.d_model;
    for (int l = c.n_layers - 1; l >= 0; --l) {
        if (c.offload_checkpoints) {
            // the layer's input comes back from the host (the top layer's is still there after a forward sweep); the
            // next layer's is requested now and travels beside this layer's sweep, into the slot of boundary l + 1
            fetch_boundary(st, l);
            wait_slot(st, l % 2);
            if (l > 0) fetch_boundary(st, l - 1);
        }
        const T *in = reinterpret_cast<const T *>(st->ckpt(l));
        float *gbuf = st->grad(l);
        st->grad_owner[st->grad_slot(l)] = -1;
        if (c.overlap) wait_grad(st, st->grad_slot(l));     // an earlier layer's Adam step may still be reading this buffer
        ensure_weights(st, l);
        prefetch_weights(st, l - 1, l);
        for (int gi = 0; gi < groups; ++gi) {
            layer_forward<T>(st, l, in + gi * gstride, nullptr);                       // recompute
            const int wb = st->plan.wgrad_groups;
            const GradStep gs{gi == 0 ? 0.f : 1.f, gi < wb ? 0.f : 1.f, gi % wb, gi % wb == wb - 1 || gi == groups - 1};
            layer_backward<T>(st, l, in + gi * gstride, dact + gi * gstride, gbuf, gs);
        }
        st->grad_owner[st->grad_slot(l)] = l;
        // update as soon as the layer's gradient is complete; in overlap mode beside the next layer's sweep
        if (fused) adam_layer(st, l, *fused, (c.overlap & LGA_OVERLAP_ADAM) != 0);
    }
    if (c.overlap) join_aux(st);                            // later work on the main stream sees every update
    if (c.offload_checkpoints) join_offload(st);
    if (dx) LGA_HIP(hipMemcpyAsync(dx, dact, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    if (fused) st->set_forward(false);                      // checkpoints no longer match the weights
    return finish("lga_backward_layered");
}

// One layer's share of the layer-major sweeps, with the layer's input (forward) and output gradient (backward)
// arriving from outside the stack: what a device of the modular pipeline (section 4) runs for each of its layers.
template <class T> int forward_layer_t(lga_stack *st, int l, const void *x_in, void *x_out) {
    const lga_config &c = st->cfg;
    const size_t act_bytes = st->T * c.d_model * sizeof(T);
    const bool offload = c.offload_checkpoints != 0;
    if (offload) {
        if (x_in == st->host_boundary(l)) {                 // the borrowed checkpoint itself: bring it back if it is away
            fetch_boundary(st, l);
            wait_slot(st, l % 2);
        } else {
            claim_slot(st, l);
            LGA_HIP(hipMemcpyAsync(st->ckpt(l), x_in, act_bytes, hipMemcpyDeviceToDevice, st->stream));
            save_boundary(st, l);
        }
        if (!x_out) claim_slot(st, l + 1);
    } else if (x_in != st->ckpt(l)) {
        LGA_HIP(hipMemcpyAsync(st->ckpt(l), x_in, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    }
    const T *in = reinterpret_cast<const T *>(st->ckpt(l));
    T *out = reinterpret_cast<T *>(x_out ? x_out : st->ckpt(l + 1));
    const int groups = c.n_micro / c.group;
    const size_t gstride = st->t * c.d_model;
    ensure_weights(st, l);
    for (int gi = 0; gi < groups; ++gi) layer_forward<T>(st, l, in + gi * gstride, out + gi * gstride);
    if (offload) {
        if (!x_out) save_boundary(st, l + 1);
        join_offload(st);
    }
    return finish("lga_forward_layer");
}

template <class T> int backward_layer_t(lga_stack *st, int l, const void *dy, void *dx, const lga_adam *fused) {
    const lga_config &c = st->cfg;
    const size_t act_bytes = st->T * c.d_model * sizeof(T);
    T *dact = st->at<T>(st->plan.dact);
    LGA_HIP(hipMemcpyAsync(dact, dy, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    const int groups = c.n_micro / c.group;
    const size_t gstride = st->t * c.d_model;
    if (c.offload_checkpoints) {
        fetch_boundary(st, l);
        wait_slot(st, l % 2);
    }
    const T *in = reinterpret_cast<const T *>(st->ckpt(l));
    st->grad_owner[st->grad_slot(l)] = -1;
    if (c.overlap) wait_grad(st, st->grad_slot(l));
    ensure_weights(st, l);
    for (int gi = 0; gi < groups; ++gi) {
        layer_forward<T>(st, l, in + gi * gstride, nullptr);                           // recompute
        const int wb = st->plan.wgrad_groups;
        const GradStep gs{gi == 0 ? 0.f : 1.f, gi < wb ? 0.f : 1.f, gi % wb, gi % wb == wb - 1 || gi == groups - 1};
        layer_backward<T>(st, l, in + gi * gstride, dact + gi * gstride, st->grad(l), gs);
    }
    st->grad_owner[st->grad_slot(l)] = l;
    if (fused) {
        adam_layer(st, l, *fused, (c.overlap & LGA_OVERLAP_ADAM) != 0);
        st->input_valid[l] = 0;
    }
    if (c.overlap) join_aux(st);
    if (dx) LGA_HIP(hipMemcpyAsync(dx, dact, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    return finish("lga_backward_layer");
}

template <class T>
int step_mbmajor_t(lga_stack *st, const void *x, const void *dy, void *y, void *dx, const lga_adam *adam) {
    const lga_config &c = st->cfg;
    const size_t act_bytes = st->T * c.d_model * sizeof(T);
    T *dact = st->at<T>(st->plan.dact);
    LGA_HIP(hipMemcpyAsync(st->ckpt(0), x, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    LGA_HIP(hipMemcpyAsync(dact, dy, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    const size_t gstride = st->t * c.d_model;               // group == 1: one micro-batch
    for (int l = 0; l < c.n_layers; ++l) st->grad_owner[l] = -1;
    for (int mu = 0; mu < c.n_micro; ++mu) {                // micro-batches outside ...
        for (int l = 0; l < c.n_layers; ++l) {              // ... layers inside
            ensure_weights(st, l);
            layer_forward<T>(st, l, reinterpret_cast<const T *>(st->ckpt(l)) + mu * gstride,
                             reinterpret_cast<T *>(st->ckpt(l + 1)) + mu * gstride);
        }
        for (int l = c.n_layers - 1; l >= 0; --l) {
            const T *in = reinterpret_cast<const T *>(st->ckpt(l)) + mu * gstride;
            ensure_weights(st, l);
            layer_forward<T>(st, l, in, nullptr);
            // layers alternate here, so every weight-gradient GEMM runs at once on its own micro-batch
            const GradStep gs{mu == 0 ? 0.f : 1.f, mu == 0 ? 0.f : 1.f, 0, true};
            layer_backward<T>(st, l, in, dact + mu * gstride, st->grad(l), gs);
        }
    }
    for (int l = 0; l < c.n_layers; ++l) st->grad_owner[l] = l;
    if (y) LGA_HIP(hipMemcpyAsync(y, st->ckpt(c.n_layers), act_bytes, hipMemcpyDeviceToDevice, st->stream));
    if (dx) LGA_HIP(hipMemcpyAsync(dx, dact, act_bytes, hipMemcpyDeviceToDevice, st->stream));
    if (adam)
        for (int l = 0; l < c.n_layers; ++l) adam_layer(st, l, *adam);
    if (c.overlap) join_aux(st);
    st->set_forward(adam == nullptr);
    return finish("lga_step_mbmajor");
}

int check_layer(const lga_stack *st, int32_t layer) {
    if (!st) return fail(LGA_ERR_ARG, "stack is NULL");
    if (layer < 0 || layer >= st->cfg.n_layers) return fail(LGA_ERR_ARG, "layer index out of range");
    return LGA_OK;
}

}  // namespace

// ==============================================================================================
extern "C" {

const char *lga_last_error(void) { return g_last_error.c_str(); }

int lga_params_per_layer(const lga_config *cfg, uint64_t *count) {
    if (!cfg || !count) return fail(LGA_ERR_ARG, "NULL argument");
    if (cfg->d_model < 1 || cfg->d_ff < 1) return fail(LGA_ERR_SHAPE, "d_model and d_ff must be >= 1");
    *count = make_layout(cfg->d_model, cfg->d_ff).total;
    return LGA_OK;
}

int lga_arena_bytes(const lga_config *cfg, uint64_t *bytes) {
    if (!bytes) return fail(LGA_ERR_ARG, "NULL argument");
    if (int rc = validate_config(cfg)) return rc;
    *bytes = make_plan(*cfg).total;
    return LGA_OK;
}

int lga_host_bytes(const lga_config *cfg, uint64_t *bytes) {
    if (!bytes) return fail(LGA_ERR_ARG, "NULL argument");
    if (int rc = validate_config(cfg)) return rc;
    const uint64_t boundary = (uint64_t)cfg->n_micro * cfg->micro_batch * cfg->seq_len * cfg->d_model *
                              (cfg->dtype != LGA_FP32 ? 2 : 4);
    *bytes = cfg->offload_checkpoints ? (uint64_t)(cfg->n_layers + 1) * boundary : 0;
    return LGA_OK;
}

int lga_traffic_model(const lga_config *cfg, int32_t order, uint64_t *param_bytes, uint64_t *grad_bytes,
                      double *flops) {
    if (int rc = validate_config(cfg)) return rc;
    if (order != LGA_ORDER_LAYERED && order != LGA_ORDER_MICROBATCH_MAJOR) return fail(LGA_ERR_ARG, "bad order");
    const LayerLayout lay = make_layout(cfg->d_model, cfg->d_ff);
    const uint64_t P = lay.total, Pm = lay.matrices, df = (uint64_t)cfg->d_model * cfg->d_ff;
    const uint64_t L = cfg->n_layers;
    const uint64_t groups = order == LGA_ORDER_LAYERED ? cfg->n_micro / cfg->group : cfg->n_micro;
    const bool is16 = cfg->dtype != LGA_FP32;
    const uint64_t wsz = is16 ? 2 : 4;
    // Adam: read w, m, v (12 B), write w, m, v (12 B) and the 16-bit copy; per group the GEMM families
    // read the matrices: forward all four, recompute all but W_2, input gradient all four.
    // the 16-bit modes also write the 16-bit copy (2 B) and re-reads / writes the matrices once for the transposed copy
    const uint64_t copies = is16 ? 2 * P + 4 * Pm : 0;
    const uint64_t per_group_param = wsz * (3 * Pm - df);
    // Restores of a steady-state step (param_buffers < n_layers): a layer's masters are cast again (read 4 B, write
    // 2 B per parameter, plus the transposed copy) whenever another layer has used its buffer since.  Counted by
    // walking the order's sequence of layer visits for two steps and keeping the second.
    const int nbuf = cfg->param_buffers ? cfg->param_buffers : cfg->n_layers;
    uint64_t restores = 0, adam_copies = L;
    if (is16 && nbuf < cfg->n_layers) {
        std::vector<int> owner(nbuf);
        for (int i = 0; i < nbuf; ++i) owner[i] = i;
        auto visit = [&](int l) {
            if (owner[l % nbuf] != l) { owner[l % nbuf] = l; ++restores; }
        };
        const int passes = order == LGA_ORDER_LAYERED ? 1 : cfg->n_micro;
        for (int step = 0; step < 2; ++step) {
            restores = 0;
            for (int pass = 0; pass < passes; ++pass) {
                for (int l = 0; l < cfg->n_layers; ++l) visit(l);
                for (int l = cfg->n_layers - 1; l >= 0; --l) visit(l);
            }
        }
        // the micro-batch-major order runs Adam for all layers at the end: only the resident ones get fresh copies
        if (order == LGA_ORDER_MICROBATCH_MAJOR) adam_copies = nbuf;
    }
    if (param_bytes)
        *param_bytes = L * (24 * P + groups * per_group_param) + adam_copies * copies + restores * (4 * P + copies);
    // gradient buffer: the first pass over it writes (4 B), later ones read-modify-write (8 B); Adam reads
    // (4 B).  Vectors take one pass per group; matrices one per weight-gradient GEMM, which in the layered
    // 16-bit path covers wgrad_groups groups.
    uint64_t mat_passes = groups;
    if (order == LGA_ORDER_LAYERED && is16) {
        const uint64_t wb = make_plan(*cfg).wgrad_groups;
        mat_passes = (groups + wb - 1) / wb;
    }
    if (grad_bytes)
        *grad_bytes = L * (4 * P + 4 * P + (groups - 1) * 8 * (P - Pm) + (mat_passes - 1) * 8 * Pm);
    if (flops) {
        const double tokens = (double)cfg->n_micro * cfg->micro_batch * cfg->seq_len;
        const double gemm = 2.0 * tokens * (double)L * (4.0 * Pm - df);                 // fwd, recompute - W_2, dX, dW
        const double seqs = (double)cfg->n_micro * cfg->micro_batch;
        // attention products executed: forward 2, recompute 2, dQ kernel 3, dK/dV kernel 4, each s^2 d_m flop with
        // the causal mask (half of the pairs are skipped), twice that without
        const double attn = (cfg->attention == LGA_ATTN_CAUSAL ? 11.0 : 22.0) * seqs * (double)L * (double)cfg->seq_len *
                            cfg->seq_len * cfg->d_model;
        *flops = gemm + attn;
    }
    return LGA_OK;
}

int lga_restore_count(lga_stack *st, uint64_t *count) {
    if (!st || !count) return fail(LGA_ERR_ARG, "NULL argument");
    *count = st->restores;
    return LGA_OK;
}

int lga_init_stack(const lga_config *cfg, const float *host_params, lga_stack **out) {
    if (!out) return fail(LGA_ERR_ARG, "out is NULL");
    *out = nullptr;
    if (int rc = validate_config(cfg)) return rc;
    {
        // dynamic-LDS limits of the large kernels, once per process and before any launch
        const hipError_t pe = prepare_kernels();
        if (pe != hipSuccess) {
            (void)hipGetLastError();
            return fail(LGA_ERR_HIP, std::string("raising the kernels' dynamic LDS limit: ") + hipGetErrorString(pe));
        }
    }
    lga_stack *st = new (std::nothrow) lga_stack();
    if (!st) return fail(LGA_ERR_OOM, "host allocation failed");
    st->cfg = *cfg;
    st->lay = make_layout(cfg->d_model, cfg->d_ff);
    st->plan = make_plan(*cfg);
    st->stream = reinterpret_cast<hipStream_t>(cfg->stream);
    st->P = st->lay.total;
    st->T = (size_t)cfg->n_micro * cfg->micro_batch * cfg->seq_len;
    st->t = (size_t)cfg->group * cfg->micro_batch * cfg->seq_len;
    st->input_valid.assign(cfg->n_layers, 0);
    st->ngrad = cfg->retain_grads ? cfg->n_layers : (cfg->overlap & LGA_OVERLAP_ADAM) ? std::min(2, cfg->n_layers) : 1;
    st->aux = nullptr;
    st->ev_fork = nullptr;
    st->host_ckpt = nullptr;
    for (int i = 0; i < 2; ++i) {
        st->dev_boundary[i] = -1;
        st->ev_ck[i] = nullptr;
        st->ck_pending[i] = 0;
    }
    st->nbuf = cfg->param_buffers ? cfg->param_buffers : cfg->n_layers;
    st->grad_owner.assign(st->ngrad, -1);
    st->w16_owner.assign(st->nbuf, -1);
    st->w16_pending.assign(st->nbuf, 0);
    st->grad_pending.assign(st->ngrad, 0);
    st->restores = 0;
    st->arena = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&st->arena), st->plan.total);
    if (e != hipSuccess) {
        std::string msg = std::string("hipMalloc of ") + std::to_string(st->plan.total) + " bytes: " + hipGetErrorString(e);
        delete st;
        (void)hipGetLastError();
        return fail(e == hipErrorOutOfMemory ? LGA_ERR_OOM : LGA_ERR_HIP, msg);
    }
    auto bail = [&](hipError_t err, const char *what) {
        std::string msg = std::string(what) + ": " + hipGetErrorString(err);
        release_stack(st);
        return fail(LGA_ERR_HIP, msg);
    };
    if (cfg->overlap || cfg->offload_checkpoints) {
        // second stream (default priority) and the event that orders it behind the main stream
        if ((e = hipStreamCreateWithFlags(&st->aux, hipStreamNonBlocking)) != hipSuccess) return bail(e, "create stream");
        if ((e = hipEventCreateWithFlags(&st->ev_fork, hipEventDisableTiming)) != hipSuccess) return bail(e, "create event");
    }
    if (cfg->offload_checkpoints) {
        // pinned (allocated as such, not registered afterwards) so that the copies run asynchronously
        const size_t bytes = (size_t)(cfg->n_layers + 1) * st->boundary_bytes();
        if ((e = hipHostMalloc(reinterpret_cast<void **>(&st->host_ckpt), bytes, hipHostMallocDefault)) != hipSuccess) {
            std::string msg = std::string("hipHostMalloc of ") + std::to_string(bytes) + " bytes: " + hipGetErrorString(e);
            release_stack(st);
            (void)hipGetLastError();
            return fail(LGA_ERR_OOM, msg);
        }
        for (auto &ev : st->ev_ck)
            if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "create event");
    }
    if (cfg->overlap) {
        st->ev_w16.assign(st->nbuf, nullptr);
        st->ev_grad.assign(st->ngrad, nullptr);
        for (auto &ev : st->ev_w16)
            if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "create event");
        for (auto &ev : st->ev_grad)
            if ((e = hipEventCreateWithFlags(&ev, hipEventDisableTiming)) != hipSuccess) return bail(e, "create event");
    }
    const size_t LP = (size_t)cfg->n_layers * st->P;
    if ((e = hipMemsetAsync(st->m(0), 0, LP * 4, st->stream)) != hipSuccess) return bail(e, "clear m");
    if ((e = hipMemsetAsync(st->v(0), 0, LP * 4, st->stream)) != hipSuccess) return bail(e, "clear v");
    if (host_params) {
        if ((e = hipMemcpyAsync(st->w(0), host_params, LP * 4, hipMemcpyHostToDevice, st->stream)) != hipSuccess)
            return bail(e, "copy parameters");
    } else {
        if ((e = hipMemsetAsync(st->w(0), 0, LP * 4, st->stream)) != hipSuccess) return bail(e, "clear w");
        const size_t d = cfg->d_model, f = cfg->d_ff;
        for (int l = 0; l < cfg->n_layers; ++l) {
            float *w = st->w(l);
            const uint64_t seed = 0x5EEDull + 16 * (uint64_t)l;
            launch_fill_const(w + st->lay.ln1_g, d, 1.0f, st->stream);
            launch_fill_const(w + st->lay.ln2_g, d, 1.0f, st->stream);
            launch_fill_normal(w + st->lay.w_qkv, d * 3 * d, 0.02f, seed + 0, st->stream);
            launch_fill_normal(w + st->lay.w_o, d * d, 0.02f, seed + 1, st->stream);
            launch_fill_normal(w + st->lay.w_1, d * f, 0.02f, seed + 2, st->stream);
            launch_fill_normal(w + st->lay.w_2, f * d, 0.02f, seed + 3, st->stream);
        }
    }
    st->cfg.overlap = 0;                                            // the initial fill runs on the main stream
    for (int l = 0; l < st->nbuf; ++l) ensure_weights(st, l);       // section 2.5: converted to 16 bits before use
    st->cfg.overlap = cfg->overlap;
    st->restores = 0;
    if ((e = hipStreamSynchronize(st->stream)) != hipSuccess) return bail(e, "init sync");
    if ((e = hipGetLastError()) != hipSuccess) return bail(e, "init kernels");
    *out = st;
    return LGA_OK;
}

void lga_destroy_stack(lga_stack *st) {
    if (!st) return;
    (void)hipStreamSynchronize(st->stream);
    release_stack(st);
}

// fn<T>(args) with T = the stack's activation type
#define LGA_DISPATCH(st, fn, ...)                                   \
    ((st)->cfg.dtype == LGA_BF16   ? fn<bf16>(__VA_ARGS__)          \
     : (st)->cfg.dtype == LGA_FP16 ? fn<f16>(__VA_ARGS__)           \
                                   : fn<float>(__VA_ARGS__))

int lga_forward_layered(lga_stack *st, const void *x, void *y) {
    if (!st || !x) return fail(LGA_ERR_ARG, "NULL argument");
    if (int rc = refuse_capture(st, "lga_forward_layered")) return rc;
    int rc = LGA_DISPATCH(st, forward_layered_t, st, x, y);
    if (rc == LGA_OK) st->set_forward(true);
    return rc;
}

int lga_backward_layered(lga_stack *st, const void *dy, void *dx, const lga_adam *fused) {
    if (!st || !dy) return fail(LGA_ERR_ARG, "NULL argument");
    if (!st->have_forward()) return fail(LGA_ERR_STATE, "lga_backward_layered needs a preceding forward pass");
    if (!fused && !st->cfg.retain_grads && st->cfg.n_layers > 1)
        return fail(LGA_ERR_STATE, "unfused backward with a single gradient buffer would lose all but one layer's gradient");
    if (fused)
        if (int rc = check_adam(fused)) return rc;
    if (int rc = refuse_capture(st, "lga_backward_layered")) return rc;
    return LGA_DISPATCH(st, backward_layered_t, st, dy, dx, fused);
}

int lga_forward_layer(lga_stack *st, int32_t layer, const void *x_in, void *x_out) {
    if (int rc = check_layer(st, layer)) return rc;
    if (!x_in) return fail(LGA_ERR_ARG, "x_in is NULL");
    if (int rc = refuse_capture(st, "lga_forward_layer")) return rc;
    int rc = LGA_DISPATCH(st, forward_layer_t, st, layer, x_in, x_out);
    if (rc == LGA_OK) {
        st->input_valid[layer] = 1;
        // the next boundary now holds this layer's output (or nothing new): not an input the next layer has seen
        if (!x_out && layer + 1 < st->cfg.n_layers) st->input_valid[layer + 1] = 0;
    }
    return rc;
}

int lga_backward_layer(lga_stack *st, int32_t layer, const void *dy, void *dx, const lga_adam *fused) {
    if (int rc = check_layer(st, layer)) return rc;
    if (!dy) return fail(LGA_ERR_ARG, "dy is NULL");
    if (!st->input_valid[layer])
        return fail(LGA_ERR_STATE, "lga_backward_layer needs a preceding forward of this layer with its current weights");
    if (fused)
        if (int rc = check_adam(fused)) return rc;
    if (int rc = refuse_capture(st, "lga_backward_layer")) return rc;
    return LGA_DISPATCH(st, backward_layer_t, st, layer, dy, dx, fused);
}

int lga_step_mbmajor(lga_stack *st, const void *x, const void *dy, void *y, void *dx, const lga_adam *adam) {
    if (!st || !x || !dy) return fail(LGA_ERR_ARG, "NULL argument");
    if (!st->cfg.retain_grads) return fail(LGA_ERR_STATE, "micro-batch-major order needs retain_grads = 1");
    if (st->cfg.group != 1) return fail(LGA_ERR_STATE, "micro-batch-major order needs group = 1");
    if (st->cfg.offload_checkpoints)
        return fail(LGA_ERR_STATE, "the micro-batch-major order keeps every boundary on the device: not available with "
                                   "offload_checkpoints");
    if (adam)
        if (int rc = check_adam(adam)) return rc;
    if (int rc = refuse_capture(st, "lga_step_mbmajor")) return rc;
    return LGA_DISPATCH(st, step_mbmajor_t, st, x, dy, y, dx, adam);
}

int lga_adam_step_layer(lga_stack *st, int32_t layer, const lga_adam *adam) {
    if (int rc = check_layer(st, layer)) return rc;
    if (!adam) return fail(LGA_ERR_ARG, "adam is NULL");
    if (int rc = check_adam(adam)) return rc;
    if (st->grad_owner[st->grad_slot(layer)] != layer)
        return fail(LGA_ERR_STATE, "no accumulated gradient is available for this layer");
    if (int rc = refuse_capture(st, "lga_adam_step_layer")) return rc;
    adam_layer(st, layer, *adam);
    st->input_valid[layer] = 0;
    return finish("lga_adam_step_layer");
}

int lga_grads(lga_stack *st, int32_t layer, const float **dev_ptr, size_t *count) {
    if (int rc = check_layer(st, layer)) return rc;
    if (!dev_ptr) return fail(LGA_ERR_ARG, "dev_ptr is NULL");
    if (st->grad_owner[st->grad_slot(layer)] != layer)
        return fail(LGA_ERR_STATE, "no accumulated gradient is available for this layer");
    *dev_ptr = st->grad(layer);
    if (count) *count = st->P;
    return LGA_OK;
}

int lga_params(lga_stack *st, int32_t layer, const float **dev_master, size_t *count) {
    if (int rc = check_layer(st, layer)) return rc;
    if (!dev_master) return fail(LGA_ERR_ARG, "dev_master is NULL");
    *dev_master = st->w(layer);
    if (count) *count = st->P;
    return LGA_OK;
}

int lga_moments(lga_stack *st, int32_t layer, float **dev_m, float **dev_v, size_t *count) {
    if (int rc = check_layer(st, layer)) return rc;
    if (dev_m) *dev_m = st->m(layer);
    if (dev_v) *dev_v = st->v(layer);
    if (count) *count = st->P;
    return LGA_OK;
}

int lga_checkpoint(lga_stack *st, int32_t boundary, const void **dev_ptr, size_t *bytes) {
    if (!st || !dev_ptr) return fail(LGA_ERR_ARG, "NULL argument");
    if (boundary < 0 || boundary > st->cfg.n_layers) return fail(LGA_ERR_ARG, "boundary index out of range");
    *dev_ptr = st->cfg.offload_checkpoints ? st->host_boundary(boundary) : st->ckpt(boundary);
    if (bytes) *bytes = st->boundary_bytes();
    return LGA_OK;
}

int lga_nonfinite_layers(lga_stack *st, int32_t *flags, int32_t *count) {
    if (!st || !count) return fail(LGA_ERR_ARG, "NULL argument");
    join_aux(st);                       // Adam steps of the overlap mode run on the second stream
    std::vector<int> host(st->cfg.n_layers);
    LGA_HIP(hipMemcpyAsync(host.data(), st->nonfinite(0), host.size() * sizeof(int), hipMemcpyDeviceToHost, st->stream));
    LGA_HIP(hipStreamSynchronize(st->stream));
    int32_t n = 0;
    for (int l = 0; l < st->cfg.n_layers; ++l) {
        n += host[l] != 0;
        if (flags) flags[l] = host[l] != 0;
    }
    *count = n;
    return LGA_OK;
}

int lga_grads_nonfinite(lga_stack *st, int32_t *flags, int32_t *count) {
    if (!st || !count) return fail(LGA_ERR_ARG, "NULL argument");
    join_aux(st);
    for (int l = 0; l < st->cfg.n_layers; ++l) {
        launch_fill_const(reinterpret_cast<float *>(st->nonfinite(l)), 1, 0.f, st->stream);
        if (st->grad_owner[st->grad_slot(l)] == l) launch_nonfinite_flag(st->grad(l), st->P, st->nonfinite(l), st->stream);
    }
    return lga_nonfinite_layers(st, flags, count);
}

int lga_loss_scaler_update(lga_loss_scaler *sc, int32_t overflowed) {
    if (!sc) return fail(LGA_ERR_ARG, "scaler is NULL");
    if (!(sc->scale > 0.f) || !(sc->growth >= 1.f) || !(sc->backoff > 0.f && sc->backoff <= 1.f) || sc->growth_interval < 1 ||
        !(sc->min_scale > 0.f) || !(sc->max_scale >= sc->min_scale) || sc->good_steps < 0)
        return fail(LGA_ERR_ARG, "loss scaler: need scale > 0, growth >= 1, 0 < backoff <= 1, growth_interval >= 1, "
                                 "0 < min_scale <= max_scale, good_steps >= 0");
    if (overflowed) {
        sc->scale = std::max(sc->scale * sc->backoff, sc->min_scale);
        sc->good_steps = 0;
    } else if (++sc->good_steps >= sc->growth_interval) {
        sc->scale = std::min(sc->scale * sc->growth, sc->max_scale);
        sc->good_steps = 0;
    }
    return LGA_OK;
}

static int profile_begin(lga_stack *st, const char *only) {
    if (!st) return fail(LGA_ERR_ARG, "stack is NULL");
    LaunchProfiler &p = profiler();
    p.only = only ? only : "";
    for (auto &r : p.records) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    p.records.clear();
    p.enabled = true;
    return LGA_OK;
}

int lga_profile_begin(lga_stack *st) { return profile_begin(st, nullptr); }
int lga_profile_begin_only(lga_stack *st, const char *kernel_name) { return profile_begin(st, kernel_name); }

int lga_profile_end(lga_stack *st, lga_kernel_stat *out, int32_t capacity, int32_t *count) {
    if (!st || !count || (capacity > 0 && !out) || capacity < 0) return fail(LGA_ERR_ARG, "bad argument");
    LaunchProfiler &p = profiler();
    p.enabled = false;
    LGA_HIP(hipStreamSynchronize(st->stream));
    std::map<std::string, lga_kernel_stat> agg;
    for (auto &r : p.records) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            lga_kernel_stat &k = agg[r.name];
            if (k.launches == 0) {
                std::memset(&k, 0, sizeof(k));
                std::strncpy(k.name, r.name.c_str(), sizeof(k.name) - 1);
            }
            k.launches += 1;
            k.ms += ms;
            k.flops += r.flops;
            k.bytes += r.bytes;
        }
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    p.records.clear();
    (void)hipGetLastError();
    std::vector<lga_kernel_stat> v;
    for (auto &kv : agg) v.push_back(kv.second);
    std::sort(v.begin(), v.end(), [](const lga_kernel_stat &a, const lga_kernel_stat &b) { return a.ms > b.ms; });
    *count = (int32_t)v.size();
    for (int32_t i = 0; i < capacity && i < (int32_t)v.size(); ++i) out[i] = v[i];
    return LGA_OK;
}

}  // extern "C"
