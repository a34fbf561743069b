"""GPU checks at the benchmark configurations' full sizes - cfg3, which bench.py times (4 layers, d = 12288,
96 heads, d_ff = 49152, seq 2048, 32 micro-batches), once more in IEEE half, and the two smaller bf16 configurations
cfg1 and cfg2 - in the launch configuration bench.py uses (layered order, the benchmark's `group` of the configuration,
single gradient buffer, fused Adam, device-filled weights).

The fp64 oracle cannot run this size, so it checks sampled outputs it can compute one by one:
attention is causal, hence the first P positions of a sequence at the first layer boundary depend
only on the first P input positions of that sequence and on layer 0's parameters.  The oracle's
layer forward on those prefixes is compared with the library's checkpoint (bf16 gate 2e-2, half precision 2.5e-3).
Beyond the samples, properties that hold at any size are checked: the whole step is reproduced
by a differently grouped run that also keeps its boundary activations in pinned host memory
(activations bit-identical, gradients equal up to fp32 re-association), and the key-bias gradient
vanishes against the query-bias gradient.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import lga_oracle as O
import synth_inputs as S
from paper_2106_02679_amd import binding as B
from gpu_helpers import rel_err

PREFIX = 48


def _run(w, group, x, dy, want_layer0_params, offload=0):
    dt = B.LGA_FP16 if w.dtype == "fp16" else B.LGA_BF16
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, dt,
                        group=group, retain_grads=0, offload_checkpoints=offload)
    st = B.Stack(cfg)
    out = {}
    try:
        if want_layer0_params:
            ptr, n = st.params(0)
            torch.cuda.synchronize()
            out["params0"] = B.read_device(ptr, n)
        st.forward_layered(x.data_ptr(), None)
        torch.cuda.synchronize()
        ptr, nbytes = st.checkpoint(1)
        d, s = w.d_model, w.seq_len
        # boundary 1, micro-batches 0 and n-1, first PREFIX positions
        samples = {}
        for mu in (0, w.n_micro - 1):
            off = mu * w.micro_batch * s * d
            bits = B.read_device(ptr + off * 2, PREFIX * d, "uint16")
            samples[mu] = S.from_16bit_bits(bits, w.dtype).astype(np.float64).reshape(PREFIX, d)
        out["samples"] = samples
        ptr, _ = st.checkpoint(w.n_layers)
        out["y_head"] = B.read_device(ptr, 4 * s * d // 4, "uint16").copy()
        st.backward_layered(dy.data_ptr(), None, B.lga_adam(1e-3, 0.9, 0.999, 1e-8, 1, 0.0, 1 if dt == B.LGA_FP16 else 0))
        torch.cuda.synchronize()
        if dt == B.LGA_FP16:
            assert st.nonfinite_layers() == [0] * w.n_layers
        ptr, n = st.grads(0)
        g0 = B.read_device(ptr, n)
        sl = S.tensor_slices(w.d_model, w.d_ff)
        out["g_ln1"] = g0[sl["ln1_g"]].copy()
        out["g_bqkv"] = g0[sl["b_qkv"]].copy()
        out["g_wo_rows"] = g0[sl["w_o"]][: 64 * d].copy()
        out["g_w2_rows"] = g0[sl["w_2"]][: 16 * d].copy()
    finally:
        st.close()
    return out


@pytest.mark.parametrize("config,dtype", [(1, "bf16"), (2, "bf16"), (3, "bf16"), (3, "fp16")])
def test_full_size_sampled_prefix_parity_and_regrouping(config, dtype):
    w = S.CONFIGS[config]
    if dtype != w.dtype:
        w = S.Workload(w.name.replace(w.dtype, dtype), w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch,
                       w.n_micro, dtype)
    tdt = torch.float16 if dtype == "fp16" else torch.bfloat16
    gate = 2.5e-3 if dtype == "fp16" else 2e-2
    free, _ = torch.cuda.mem_get_info()
    need = B.arena_bytes(B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro,
                                       B.LGA_BF16, group=S.BENCH_GROUP[config])) + 6 * w.tokens * w.d_model * 2 + 4e9
    if free < need:
        pytest.skip(f"needs about {need / 1e9:.0f} GB of free HBM")
    shape = (w.n_micro, w.micro_batch, w.seq_len, w.d_model)
    gen = torch.Generator(device="cuda").manual_seed(0)
    x = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(tdt)
    dy = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(tdt)
    a = _run(w, S.BENCH_GROUP[config], x, dy, True)
    # --- sampled outputs against the oracle
    p0 = O.unflatten_layer(a["params0"], w.d_model, w.d_ff)
    a["params0"] = None
    for mu, got in a["samples"].items():
        xin = x[mu, 0, :PREFIX].float().cpu().numpy().astype(np.float64)[None]
        ref, _ = O.layer_forward(xin, p0, w.n_heads, 1e-5)
        err = rel_err(got, ref[0])
        print(f"{w.name} boundary 1, micro-batch {mu}, first {PREFIX} positions: rel err {err:.3e}")
        assert err < gate
    del p0
    # --- the degenerate key-bias gradient
    d = w.d_model
    assert np.linalg.norm(a["g_bqkv"][d:2 * d]) < 5e-2 * np.linalg.norm(a["g_bqkv"][:d])
    # --- same step with another grouping (same kernels per token, different fp32 summation order) and with the
    # boundary activations offloaded to the host (1.6 GB per boundary, read back from there)
    b = _run(w, S.BENCH_GROUP[config] // 2, x, dy, False, offload=1)
    assert np.array_equal(a["y_head"], b["y_head"])
    for mu in a["samples"]:
        assert np.array_equal(a["samples"][mu], b["samples"][mu])
    for key in ("g_ln1", "g_bqkv", "g_wo_rows", "g_w2_rows"):
        assert rel_err(b[key], a[key]) < 1e-4, key


# ---------------------------------------------------------------------------------------------------------------
# Gradients and the Adam step at full size, against the oracle.
#
# One layer at the configuration's full width, micro-batch count and grouping - the launch configuration of the
# benchmark: every GEMM has its full tile grid and the merged weight-gradient GEMMs contract over all of the step's
# tokens.  The output gradient is zero except on the first PREFIX_G positions of a few sequences spread over the
# micro-batches.  With the causal mask nothing outside those prefixes can contribute: the layer's backward pass is
# row-wise except for attention, where a key or value position only hears from queries at or after it, so every
# activation gradient vanishes outside the prefixes, and every weight gradient is a sum over the prefix tokens alone,
# whose activations depend only on the prefixes of x.  The oracle's layer_forward / layer_backward on the prefixes
# (as one batch of short sequences; micro-batch gradients add, section 2.5) therefore give every weight gradient of
# the full-size step exactly.  A second backward pass with a dense output gradient adds the checks that have a
# closed form at any size: the last linear map's bias gradient is the column sum of dy over all tokens, and the Adam
# step maps (w, m = 0, v = 0, g) to its closed form element by element.
PREFIX_G = 72          # crosses the 64-element k tile of the weight-gradient GEMMs


def bf16_gate(w):
    """The bf16 gate of 2e-2, widened where the workload's own initialisation makes the softmax ill-conditioned.
    q and k are stored in bf16 (rms relative rounding error about 1.6e-3 each, and as much again inherited from the
    bf16 LayerNorm output they are computed from), so a score s carries an absolute error of about 3.2e-3 |s|; the
    softmax turns an absolute score error into a relative error of the probability, and everything downstream of the
    attention output inherits it.  With weights ~ N(0, 0.02^2) and unit-variance LayerNorm outputs the scores have
    standard deviation d_m * 0.02^2: 0.3 at cfg1, 4.9 at cfg3, 10.2 at cfg4 - i.e. about 1.6e-2 and 3.3e-2 of
    relative error at the two wide configurations (measured: 1.7e-2 and 3.1e-2).  Gate: max(2e-2, 4e-3 * that
    spread), which is 2e-2 for every configuration but cfg4 (4.1e-2)."""
    return max(2e-2, 4e-3 * w.d_model * 0.02 ** 2)


def _progress(capfd, msg):
    with capfd.disabled():
        print(f"  [full-size] {msg}", flush=True)


def _chunked_rel_err(got32, ref64, chunk=1 << 26):
    """||got - ref|| / ||ref|| without array-sized temporaries (flat views)."""
    a, r = got32.reshape(-1), ref64.reshape(-1)
    num = den = 0.0
    for i in range(0, r.size, chunk):
        d = a[i:i + chunk].astype(np.float64) - r[i:i + chunk]
        num += float(d @ d)
        den += float(r[i:i + chunk] @ r[i:i + chunk])
    return (num / den) ** 0.5 if den > 0 else num ** 0.5


@pytest.mark.timeout(1200)
@pytest.mark.parametrize("config", [3, 4])
def test_full_size_weight_gradients_and_adam_against_the_oracle(config, capfd):
    base = S.CONFIGS[config]
    w = S.Workload(base.name + "_one_layer", 1, base.d_model, base.n_heads, base.d_ff, base.seq_len, base.micro_batch,
                   base.n_micro, base.dtype)
    d, f, s, n = w.d_model, w.d_ff, w.seq_len, w.n_micro
    cfg = B.make_config(1, d, w.n_heads, f, s, w.micro_batch, n, B.LGA_BF16, group=S.BENCH_GROUP[config], retain_grads=0)
    free, _ = torch.cuda.mem_get_info()
    need = B.arena_bytes(cfg) + 5 * w.tokens * d * 2 + 4e9
    if free < need:
        pytest.skip(f"needs about {need / 1e9:.0f} GB of free HBM")
    shape = (n, w.micro_batch, s, d)
    gen = torch.Generator(device="cuda").manual_seed(11 + config)
    x = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(torch.bfloat16)
    dy_dense = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(torch.bfloat16)
    # sequences spread over the groups and over the merged weight-gradient GEMMs (cfg4 runs three of them per step)
    picked = sorted({0, 5, (2 * n) // 5, (2 * n) // 3, n - 1}) if config == 3 else [0, n // 2 - 3, n - 1]
    dy_sparse = torch.zeros_like(dy_dense)
    for mu in picked:
        dy_sparse[mu, 0, :PREFIX_G] = dy_dense[mu, 0, :PREFIX_G]
    sl = S.tensor_slices(d, f)
    shapes = S.tensor_shapes(d, f)
    st = B.Stack(cfg)
    try:
        # ---- sparse output gradient: every weight gradient against the oracle
        st.forward_layered(x.data_ptr(), None)
        st.backward_layered(dy_sparse.data_ptr(), None, None)
        torch.cuda.synchronize()
        _progress(capfd, f"{w.name}: GPU step done, reading layer parameters")
        wptr, P = st.params(0)
        p = {name: B.read_device(wptr + 4 * sl[name].start, sl[name].stop - sl[name].start).astype(np.float64).reshape(shapes[name])
             for name in S.PARAM_ORDER}
        xs = np.stack([x[mu, 0, :PREFIX_G].float().cpu().numpy().astype(np.float64) for mu in picked])
        gs = np.stack([dy_sparse[mu, 0, :PREFIX_G].float().cpu().numpy().astype(np.float64) for mu in picked])
        _progress(capfd, f"oracle forward on {len(picked)} prefixes of {PREFIX_G} positions")
        y_ref, cache = O.layer_forward(xs, p, w.n_heads, 1e-5)
        cptr, _ = st.checkpoint(1)
        for i, mu in enumerate(picked):
            bits = B.read_device(cptr + 2 * mu * w.micro_batch * s * d, PREFIX_G * d, "uint16")
            got = S.from_16bit_bits(bits, "bf16").astype(np.float64).reshape(PREFIX_G, d)
            err = rel_err(got, y_ref[i])
            assert err < 2e-2, (mu, err)
        gate = bf16_gate(w)
        _progress(capfd, f"oracle backward (gradient gate {gate:.2e})")
        _, g_ref = O.layer_backward(gs, cache, p, w.n_heads)
        del cache, p
        gptr, _ = st.grads(0)
        worst = {}
        for name in S.PARAM_ORDER:
            got = B.read_device(gptr + 4 * sl[name].start, sl[name].stop - sl[name].start)
            worst[name] = _chunked_rel_err(got, g_ref.pop(name))
            del got
            _progress(capfd, f"gradient {name}: relative error {worst[name]:.3e}")
        bad = {k: v for k, v in worst.items() if not v < gate}
        assert not bad, bad
        assert worst["b_2"] < 1e-6 and worst["w_2"] < 2e-2            # not (b_2) or least (w_2) affected by the softmax

        # ---- dense output gradient: the closed forms
        st.backward_layered(dy_dense.data_ptr(), None, None)          # same checkpoints, weights unchanged
        torch.cuda.synchronize()
        b2 = B.read_device(gptr + 4 * sl["b_2"].start, d).astype(np.float64)
        colsum = np.zeros(d)
        flat = dy_dense.view(-1, d)
        for i in range(0, flat.shape[0], 8192):
            colsum += flat[i:i + 8192].float().cpu().numpy().astype(np.float64).sum(0)
        err = rel_err(b2, colsum)
        _progress(capfd, f"dense b_2 gradient against the fp64 column sum of dy over {flat.shape[0]} tokens: {err:.3e}")
        assert err < 1e-5                                              # fp32 sums of exactly representable inputs
        # sampled stretches of the flat vector through the Adam step
        rng = np.random.default_rng(config)
        starts = sorted(int(v) for v in rng.integers(0, P - 4096, size=48)) + [0, P - 4096, sl["w_1"].start, sl["b_qkv"].start]
        before = [(B.read_device(wptr + 4 * o, 4096).astype(np.float64), B.read_device(gptr + 4 * o, 4096).astype(np.float64))
                  for o in starts]
        adam = B.lga_adam(1e-3, 0.9, 0.999, 1e-8, 1, 0.0, 0)
        st.adam_step_layer(0, adam)
        torch.cuda.synchronize()
        mptr, vptr, _ = st.moments(0)
        from gpu_helpers import oracle_adam
        hp = oracle_adam(adam)
        for o, (w0, g0) in zip(starts, before):
            w_ref, m_ref, v_ref = O.adam_update(w0, np.zeros_like(w0), np.zeros_like(w0), g0, hp)
            assert rel_err(B.read_device(mptr + 4 * o, 4096), m_ref) < 1e-6, o
            assert rel_err(B.read_device(vptr + 4 * o, 4096), v_ref) < 1e-6, o
            # the step is lr g / (|g| + eps): compare the update itself, not the weight it is added to
            got_dw = B.read_device(wptr + 4 * o, 4096).astype(np.float64) - w0
            nz = np.abs(g0) > 1e-4                                      # away from g = 0, where the step is smooth
            assert np.abs(got_dw[nz] - (w_ref - w0)[nz]).max() < 2e-7, o          # fp32 rounding of w ~ 0.02 .. 1
            assert np.abs(got_dw).max() <= 1e-3 * (1 + 1e-3)
        _progress(capfd, "Adam closed form on sampled stretches: ok")
    finally:
        st.close()


@pytest.mark.timeout(900)
def test_cfg1_at_full_size_against_the_oracle(capfd):
    """GPT-2-small shape, all 12 layers, 8 micro-batches of 4 sequences of 1024 positions: the whole step of the
    benchmark's launch configuration (layered order, all 8 micro-batches per launch, fused per-layer Adam) against the oracle's plain
    micro-batch-major step - every boundary, every gradient tensor, the updated weights and moments."""
    from gpu_helpers import run_gpu_step, oracle_shape, adam_struct, oracle_adam, compare_with_oracle
    w = S.CONFIGS[1]
    x, G, params = S.make_inputs(w, seed=0)
    adam = adam_struct()
    _progress(capfd, f"{w.name}: oracle step over {w.tokens} tokens x {w.n_layers} layers")
    ref = O.step_microbatch_major(x, G, params, oracle_shape(w), oracle_adam(adam))
    _progress(capfd, "oracle done, GPU step")
    got = run_gpu_step(w, x, G, params, group=S.BENCH_GROUP[1], retain=1, adam=adam)
    worst = compare_with_oracle(w, got, ref, 2e-2, adam)
    top = sorted(worst.items(), key=lambda kv: -kv[1])[:5]
    _progress(capfd, "worst relative errors: " + ", ".join(f"{k} {v:.2e}" for k, v in top))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("M,N,K", [(12288, 12288, 65536), (12288, 36864, 65536), (25600, 25600, 49152)])
def test_full_size_weight_gradient_gemm_sampled_against_fp64_dot_products(M, N, K, capfd):
    """The merged weight-gradient GEMM as the benchmark configurations launch it (both operands k-contiguous with the
    stack's row pitch of K + 64, fp32 result, beta 0 then 1) on dense random operands: cfg3's out-projection and QKV
    shapes over all 65 536 tokens of a step (tile grids of whole 16 x 16 blocks: the block-wise workgroup order), and
    cfg4's out-projection shape over 49 152 (a 100 x 100 grid: the row-group order).  289 output entries - rows and
    columns at the corners, on both sides of tile boundaries and at random places - against fp64 dot products.
    Tolerance: the operands are exact in bf16 and their products exact in fp32, so the error is that of the fp32
    accumulation over K terms, about 2^-24 sqrt(K / 16) ~ 4e-6 relative for sums of random signs; gate 5e-5."""
    pitch = K + 64
    free, _ = torch.cuda.mem_get_info()
    if free < (M + N) * pitch * 2 * 3 + M * N * 4 + 2e9:
        pytest.skip("not enough free HBM")
    gen = torch.Generator(device="cuda").manual_seed(M + N + K)
    A = torch.empty((M, pitch), device="cuda", dtype=torch.bfloat16)
    Bm = torch.empty((N, pitch), device="cuda", dtype=torch.bfloat16)
    for t in (A, Bm):
        for i in range(0, t.shape[0], 4096):                     # in pieces: the fp32 temporaries stay small
            t[i:i + 4096] = torch.randn((min(4096, t.shape[0] - i), pitch), device="cuda", generator=gen).to(torch.bfloat16)
    out = torch.full((M, N), float("nan"), device="cuda", dtype=torch.float32)
    rng = np.random.default_rng(K)

    def picks(n):
        fixed = [0, 1, 255, 256, 257, n // 2 + 3, n - 257, n - 256, n - 1]
        return sorted(set(fixed + [int(v) for v in rng.integers(0, n, size=17 - len(fixed))]))

    rows, cols = picks(M), picks(N)
    a = A[rows, :K].float().cpu().numpy().astype(np.float64)
    b = Bm[cols, :K].float().cpu().numpy().astype(np.float64)
    ref = a @ b.T
    for beta, scale in ((0.0, 1.0), (1.0, 2.0)):
        B.check(B.lib.lga_op_gemm(B.LGA_BF16, 1, 1, B.LGA_EPI_ACCUM_F32, M, N, K, A.data_ptr(), pitch, Bm.data_ptr(), pitch,
                                  None, None, out.data_ptr(), N, None, None, beta, None))
        torch.cuda.synchronize()
        got = out[rows][:, cols].cpu().numpy().astype(np.float64)
        err = rel_err(got, scale * ref)
        _progress(capfd, f"weight-gradient GEMM {M} x {N} x {K}, beta {beta}: sampled relative error {err:.3e}")
        assert err < 5e-5
    assert bool(torch.isfinite(out).all())                       # every entry was written
