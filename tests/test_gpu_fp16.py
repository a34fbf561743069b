"""GPU parity of the half-precision mode (LGA_FP16) with gradient scaling (section 2.2: half precision has a
narrow exponent range, so the gradients are scaled dynamically; bfloat16 is the format that does not need it).

The kernels are the bf16 mode's with the other matrix instruction and conversion, so the gate is the bf16 gate
scaled by the ratio of the unit roundoffs, 2^-11 / 2^-8:  2e-2 / 8 = 2.5e-3, on the same tensors.

Both sides get the same output gradient dy = half(G * loss_scale), rounded on the CPU; the oracle divides by the
scale in Adam like the library does.  Overflow decisions are compared only where fp64 can know them: an output
gradient that is already infinite in half precision, and a stack whose weights are built so that one layer's
backward pass overflows by orders of magnitude while the layer above it stays small.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import lga_oracle as O
import synth_inputs as S
from paper_2106_02679_amd import binding as B
from gpu_helpers import (run_gpu_step, oracle_shape, adam_struct, oracle_adam, rel_err, to_dev, empty_dev, to_host,
                         compare_with_oracle)

GATE_FP16 = 2.5e-3


def scaled(G, scale):
    """The output gradient the caller hands over: G * scale rounded to half precision (inf where it overflows)."""
    with np.errstate(over="ignore"):
        return (G.astype(np.float64) * scale).astype(np.float16).astype(np.float32)


@pytest.mark.parametrize("dh,group,scale", [(32, 1, 0.0), (32, 4, 256.0), (64, 2, 1024.0), (128, 1, 64.0), (160, 2, 3.0),
                                            (24, 2, 128.0)])
def test_fp16_small_stacks_match_oracle(dh, group, scale):
    heads = 2
    d = heads * dh
    w = S.Workload(f"small_fp16_dh{dh}", 2, d, heads, 4 * d, 96, 2, 4, "fp16")
    x, G, params = S.make_inputs(w, seed=5)
    Gs = scaled(G, scale or 1.0)
    assert np.isfinite(Gs).all()
    adam = adam_struct(loss_scale=scale, skip_nonfinite=1 if scale else 0)
    ref = O.step_microbatch_major(x, Gs, params, oracle_shape(w), oracle_adam(adam))
    got = run_gpu_step(w, x, Gs, params, group=group, retain=1, adam=adam)
    worst = compare_with_oracle(w, got, ref, GATE_FP16, adam)
    if scale:
        assert got["skipped"] == [0, 0] and ref.skipped == [False, False]
    print(f"fp16 dh={dh} group={group} scale={scale}: worst rel err {max(worst.values()):.3e}")


def test_fp16_encoder_and_orders_agree():
    w = S.Workload("fp16_enc", 3, 128, 2, 512, 72, 1, 4, "fp16")
    x, G, params = S.make_inputs(w, seed=9, weight_std=0.05, bias_std=0.05)
    Gs = scaled(G, 512.0)
    # Adam's first step moves every entry by lr * sign(g): one sign flip of a near-zero gradient in a 128-entry bias
    # of size 0.05 costs 2 lr / 0.57 whatever the precision, so lr is kept small against this mode's gate
    adam = adam_struct(lr=1e-4, loss_scale=512.0, skip_nonfinite=1)
    ref = O.step_microbatch_major(x, Gs, params, oracle_shape(w, causal=False), oracle_adam(adam))
    lay = run_gpu_step(w, x, Gs, params, group=2, retain=1, adam=adam, attention=B.LGA_ATTN_FULL)
    compare_with_oracle(w, lay, ref, GATE_FP16, adam, zero_init=False)
    mb = run_gpu_step(w, x, Gs, params, group=1, retain=1, adam=adam, order="mbmajor", attention=B.LGA_ATTN_FULL)
    compare_with_oracle(w, mb, ref, GATE_FP16, adam, zero_init=False)
    assert np.array_equal(lay["y"], mb["y"])            # same kernels per token in either order
    tight = run_gpu_step(w, x, Gs, params, group=2, retain=0, adam=adam, attention=B.LGA_ATTN_FULL, param_buffers=2,
                         overlap=3, offload=1)
    assert np.array_equal(tight["y"], lay["y"]) and np.array_equal(tight["dx"], lay["dx"])
    for l in range(w.n_layers):
        assert np.array_equal(tight["params"][l], lay["params"][l])


def test_dynamic_loss_scale_over_three_steps_matches_oracle():
    """Step 1 at a scale that makes the output gradient itself infinite in half precision: every layer's update is
    left out on both sides.  The scaler backs off (by 2^-10, so that one back-off is enough), steps 2 and 3 go
    through; Adam's step count advances only with applied updates."""
    w = S.Workload("fp16_steps", 2, 64, 2, 256, 40, 2, 2, "fp16")
    x, G, params = S.make_inputs(w, seed=43, weight_std=0.05, bias_std=0.05)
    shape = oracle_shape(w)
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, B.LGA_FP16,
                        group=2, retain_grads=1)
    st = B.Stack(cfg, np.concatenate(params))
    sc_gpu = B.lga_loss_scaler(2.0 ** 20, 2.0, 2.0 ** -10, 1.0, 2.0 ** 24, 2, 0)
    sc_ref = O.LossScaler(scale=2.0 ** 20, growth=2.0, backoff=2.0 ** -10, growth_interval=2)
    import ctypes as C
    p, m, v = [q.astype(np.float64) for q in params], None, None
    t_gpu = t_ref = 1
    history = []
    try:
        xd = to_dev(x, B.LGA_FP16)
        yd, dxd = empty_dev(x.shape, B.LGA_FP16), empty_dev(x.shape, B.LGA_FP16)
        for step in range(4):
            assert sc_gpu.scale == sc_ref.scale
            Gs = scaled(G, sc_ref.scale)
            # --- oracle
            hp = O.AdamHyper(lr=float(np.float32(2e-3)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)),
                             eps=float(np.float32(1e-8)), step=t_ref, loss_scale=sc_ref.scale, skip_nonfinite=True)
            with np.errstate(invalid="ignore", over="ignore"):
                ref = O.step_microbatch_major(x, Gs, p, shape, hp, m, v)
            over_ref = any(ref.skipped)
            assert over_ref == all(ref.skipped)
            p, m, v = ref.new_params, ref.new_m, ref.new_v
            O.loss_scaler_update(sc_ref, over_ref)
            t_ref += 0 if over_ref else 1
            # --- library
            Gd = to_dev(Gs, B.LGA_FP16)
            st.forward_layered(xd.data_ptr(), yd.data_ptr())
            st.backward_layered(Gd.data_ptr(), dxd.data_ptr(), adam_struct(lr=2e-3, step=t_gpu, loss_scale=sc_gpu.scale,
                                                                           skip_nonfinite=1))
            flags = st.nonfinite_layers()
            over_gpu = any(flags)
            B.check(B.lib.lga_loss_scaler_update(C.byref(sc_gpu), int(over_gpu)))
            t_gpu += 0 if over_gpu else 1
            history.append((over_ref, flags))
            assert over_gpu == over_ref and flags == [int(s) for s in ref.skipped], history
        assert [h[0] for h in history] == [True, False, False, False]
        assert sc_gpu.scale == 2.0 ** 11 and t_gpu == 4            # one back-off, one growth after two clean steps
        keep = np.ones(w.params_per_layer, dtype=bool)
        sl = S.tensor_slices(w.d_model, w.d_ff)
        keep[sl["b_qkv"].start + w.d_model: sl["b_qkv"].start + 2 * w.d_model] = False
        for l in range(w.n_layers):
            ptr, n = st.params(l)
            mp, vp, _ = st.moments(l)
            assert rel_err(B.read_device(ptr, n)[keep], p[l][keep]) < GATE_FP16
            assert rel_err(B.read_device(mp, n), m[l]) < GATE_FP16
            assert 0.5 * rel_err(B.read_device(vp, n), v[l]) < GATE_FP16
    finally:
        st.close()


def test_an_overflow_inside_a_lower_layer_leaves_out_that_layer_only():
    """Layer 0's second feed-forward matrix is made so large (entries around +-300) that the input-gradient product
    through it overflows half precision by a factor of several - dy W_2^T sums 64 terms of size ~ scale * 300 - while
    its forward output and everything in layer 1 stay far inside the range.  The fused per-layer update therefore
    applies layer 1's step (compared with the oracle, whose fp64 gradient for that layer is unaffected) and leaves
    layer 0 exactly as it was; an unfused pass with retained gradients reports the same layers before any update."""
    w = S.Workload("fp16_overflow", 2, 64, 2, 256, 32, 2, 2, "fp16")
    x, G, params = S.make_inputs(w, seed=77)
    sl = S.tensor_slices(w.d_model, w.d_ff)
    rng = np.random.default_rng(1)
    params[0][sl["w_2"]] = (300.0 * rng.choice([-1.0, 1.0], size=w.d_ff * w.d_model)).astype(np.float32)
    scale = 1024.0
    Gs = scaled(G, scale)
    adam = adam_struct(loss_scale=scale, skip_nonfinite=1)
    with np.errstate(invalid="ignore", over="ignore"):
        ref = O.step_microbatch_major(x, Gs, params, oracle_shape(w), oracle_adam(adam))
    assert ref.skipped == [False, False]                   # fp64 does not overflow: the oracle applies both
    # the size argument, on the oracle's numbers: layer 0's pre-GELU gradient would need about this much range
    need = np.abs(Gs.reshape(-1, w.d_model).astype(np.float64) @ params[0][sl["w_2"]].reshape(w.d_ff, w.d_model).T.astype(np.float64)).max()
    assert need > 4 * 65504.0
    assert np.abs(ref.boundaries).max() < 0.5 * 65504.0
    got = run_gpu_step(w, x, Gs, params, group=1, retain=1, adam=adam)
    assert got["skipped"] == [1, 0]
    assert np.array_equal(got["params"][0], params[0].astype(np.float64))
    assert not got["m"][0].any() and not got["v"][0].any()
    assert not np.isfinite(got["grads"][0]).all() and np.isfinite(got["grads"][1]).all()
    keep = np.ones(w.params_per_layer, dtype=bool)
    keep[sl["b_qkv"].start + w.d_model: sl["b_qkv"].start + 2 * w.d_model] = False
    assert rel_err(got["params"][1][keep], ref.new_params[1][keep]) < GATE_FP16
    assert rel_err(got["m"][1], ref.new_m[1]) < GATE_FP16
    assert rel_err(got["boundaries"], ref.boundaries) < GATE_FP16
    # all-or-nothing variant: unfused backward, ask before updating anything
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, B.LGA_FP16,
                        group=2, retain_grads=1)
    st = B.Stack(cfg, np.concatenate(params))
    try:
        xd, Gd = to_dev(x, B.LGA_FP16), to_dev(Gs, B.LGA_FP16)
        st.forward_layered(xd.data_ptr(), None)
        st.backward_layered(Gd.data_ptr(), None, None)
        assert st.grads_nonfinite() == [1, 0]
        assert st.nonfinite_layers() == [1, 0]
        for l in range(w.n_layers):
            ptr, n = st.params(l)
            assert np.array_equal(B.read_device(ptr, n), params[l])
    finally:
        st.close()


def test_loss_scale_without_the_test_and_bad_arguments():
    w = S.Workload("fp16_args", 1, 64, 2, 256, 16, 1, 2, "fp16")
    x, G, params = S.make_inputs(w, seed=3)
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, B.LGA_FP16,
                        group=1, retain_grads=0)
    st = B.Stack(cfg, np.concatenate(params))
    try:
        xd, Gd = to_dev(x, B.LGA_FP16), to_dev(scaled(G, 8.0), B.LGA_FP16)
        st.forward_layered(xd.data_ptr(), None)
        for bad in (adam_struct(loss_scale=-1.0), adam_struct(loss_scale=float("nan")), adam_struct(loss_scale=float("inf")),
                    adam_struct(skip_nonfinite=2)):
            with pytest.raises(B.LgaError) as e:
                st.backward_layered(Gd.data_ptr(), None, bad)
            assert e.value.code == B.LGA_ERR_ARG
        st.backward_layered(Gd.data_ptr(), None, adam_struct(loss_scale=8.0))
        assert st.nonfinite_layers() == [0]                 # never tested: reported as clean
        ref = O.step_microbatch_major(x, scaled(G, 8.0), params, oracle_shape(w),
                                      oracle_adam(adam_struct(loss_scale=8.0)))
        ptr, n = st.params(0)
        keep = np.ones(w.params_per_layer, dtype=bool)
        sl = S.tensor_slices(w.d_model, w.d_ff)
        keep[sl["b_qkv"].start + w.d_model: sl["b_qkv"].start + 2 * w.d_model] = False
        assert rel_err(B.read_device(ptr, n)[keep], ref.new_params[0][keep]) < GATE_FP16
    finally:
        st.close()
