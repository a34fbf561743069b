"""GPU tests of the per-layer entry points (lga_forward_layer / lga_backward_layer): one layer's share of the
layer-major sweeps with its input and output gradient arriving from outside the stack, as on a device of the
modular pipeline (section 4), where the layers a device holds are not neighbours.

  * chained over layers 0 .. L-1 and back they reproduce lga_forward_layered / lga_backward_layered bit for bit;
  * fed with unrelated inputs per layer, in an interleaved order, each layer matches the fp64 oracle's
    one-layer step on that input (fp32 gate 1e-5, bf16 gate 2e-2);
  * the call-order rules are enforced on the host.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import lga_oracle as O
import synth_inputs as S
from paper_2106_02679_amd import binding as B
from gpu_helpers import (run_gpu_step, adam_struct, oracle_adam, rel_err, to_dev, empty_dev, to_host, dtype_code,
                         updatable_mask)

GATE = {"fp32": 1e-5, "bf16": 2e-2}


def _read_layer_state(st, l):
    ptr, n = st.params(l)
    mp, vp, _ = st.moments(l)
    return [B.read_device(p, n).copy() for p in (ptr, mp, vp)]


@pytest.mark.parametrize("dtype,via_checkpoints,offload", [("fp32", False, 0), ("bf16", False, 0), ("bf16", True, 0),
                                                           ("bf16", False, 1), ("bf16", True, 1)])
def test_per_layer_calls_chain_to_the_sweeps(dtype, via_checkpoints, offload):
    w = S.Workload("chain", 3, 128, 4, 512, 80, 1, 4, dtype)
    x, G, params = S.make_inputs(w, seed=31)
    adam = adam_struct()
    base = run_gpu_step(w, x, G, params, group=2, retain=0, adam=adam)
    dt = dtype_code(w)
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, dt, group=2,
                        retain_grads=0, offload_checkpoints=offload)
    st = B.Stack(cfg, np.concatenate(params))
    try:
        cur, nxt = to_dev(x, dt), empty_dev(x.shape, dt)
        for l in range(w.n_layers):
            if via_checkpoints:      # stay inside the library's boundaries: no activation copies at all
                src = cur.data_ptr() if l == 0 else st.checkpoint(l)[0]
                st.forward_layer(l, src, None)
            else:
                st.forward_layer(l, cur.data_ptr(), nxt.data_ptr())
                cur, nxt = nxt, cur
        torch.cuda.synchronize()
        if via_checkpoints:
            ptr, _ = st.checkpoint(w.n_layers)
            n_act = int(np.prod(x.shape))
            y = S.from_bf16_bits(B.read_device(ptr, n_act, "uint16")).astype(np.float64).reshape(x.shape)
        else:
            y = to_host(cur)
        assert np.array_equal(y, base["y"])
        dcur, dnxt = to_dev(G, dt), empty_dev(x.shape, dt)
        for l in reversed(range(w.n_layers)):
            st.backward_layer(l, dcur.data_ptr(), dnxt.data_ptr(), adam)
            dcur, dnxt = dnxt, dcur
        torch.cuda.synchronize()
        assert np.array_equal(to_host(dcur), base["dx"])
        ptr, n = st.grads(0)
        assert np.array_equal(B.read_device(ptr, n).astype(np.float64), base["grads"][0])
        for l in range(w.n_layers):
            wl, ml, vl = _read_layer_state(st, l)
            assert np.array_equal(wl.astype(np.float64), base["params"][l]), l
            assert np.array_equal(ml.astype(np.float64), base["m"][l]), l
            assert np.array_equal(vl.astype(np.float64), base["v"][l]), l
    finally:
        st.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_layers_with_outside_inputs_match_one_layer_oracle_steps(dtype):
    """Two layers of one stack used as a modular layer set: each gets its own input and output gradient, the calls
    interleave, one layer updates through the fused path and the other through lga_adam_step_layer."""
    w = S.Workload("modular", 2, 96, 3, 384, 72, 2, 2, dtype)
    one = S.Workload("modular1", 1, 96, 3, 384, 72, 2, 2, dtype)
    x0, G0, params = S.make_inputs(w, seed=41, weight_std=0.05, bias_std=0.05)
    x1, G1, _ = S.make_inputs(one, seed=42)
    adam = adam_struct(lr=3e-3, step=2)
    shape1 = O.StackShape(d_l=1, d_m=w.d_model, d_a=w.n_heads, d_I=w.d_ff, d_s=w.seq_len, b_mu=w.micro_batch,
                          n_mu=w.n_micro)
    refs = [O.step_microbatch_major(xi, Gi, [params[l]], shape1, oracle_adam(adam))
            for l, (xi, Gi) in enumerate(((x0, G0), (x1, G1)))]
    dt = dtype_code(w)
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, dt, group=1,
                        retain_grads=0)
    st = B.Stack(cfg, np.concatenate(params))
    gate = GATE[dtype]
    keep = updatable_mask(w)
    try:
        xin = [to_dev(x0, dt), to_dev(x1, dt)]
        dys = [to_dev(G0, dt), to_dev(G1, dt)]
        outs = [empty_dev(x0.shape, dt) for _ in range(2)]
        dxs = [empty_dev(x0.shape, dt) for _ in range(2)]
        st.forward_layer(1, xin[1].data_ptr(), outs[1].data_ptr())
        st.forward_layer(0, xin[0].data_ptr(), outs[0].data_ptr())
        # layer 1: unfused backward, gradient read back, then its own Adam call
        st.backward_layer(1, dys[1].data_ptr(), dxs[1].data_ptr(), None)
        torch.cuda.synchronize()
        ptr, n = st.grads(1)
        g1 = B.read_device(ptr, n).astype(np.float64)
        st.adam_step_layer(1, adam)
        # layer 0: fused
        st.backward_layer(0, dys[0].data_ptr(), dxs[0].data_ptr(), adam)
        torch.cuda.synchronize()
        ptr, n = st.grads(0)
        g0 = B.read_device(ptr, n).astype(np.float64)
        with pytest.raises(B.LgaError):
            st.grads(1)                      # the single gradient buffer now holds layer 0's
        for l, g in ((0, g0), (1, g1)):
            ref = refs[l]
            assert rel_err(to_host(outs[l]), ref.boundaries[1]) < gate, l
            assert rel_err(to_host(dxs[l]), ref.dx) < gate, l
            sl = S.tensor_slices(w.d_model, w.d_ff)
            for name in S.PARAM_ORDER:
                if name == "b_qkv":          # its key third is identically zero: compare the rest
                    d = w.d_model
                    got_b = np.concatenate([g[sl[name]][:d], g[sl[name]][2 * d:]])
                    ref_b = np.concatenate([ref.grads[0][sl[name]][:d], ref.grads[0][sl[name]][2 * d:]])
                    assert rel_err(got_b, ref_b) < gate, (l, name)
                else:
                    assert rel_err(g[sl[name]], ref.grads[0][sl[name]]) < gate, (l, name)
            wl, ml, vl = _read_layer_state(st, l)
            assert rel_err(wl[keep], ref.new_params[0][keep]) < gate, l
            assert rel_err(ml, ref.new_m[0]) < gate, l
            assert 0.5 * rel_err(vl, ref.new_v[0]) < gate, l
    finally:
        st.close()


def test_per_layer_call_order_rules():
    w = S.Workload("rules", 2, 64, 2, 256, 32, 1, 2, "bf16")
    x, G, params = S.make_inputs(w, seed=3)
    dt = dtype_code(w)
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, dt, group=1,
                        retain_grads=0)
    st = B.Stack(cfg, np.concatenate(params))
    xd, Gd, out = to_dev(x, dt), to_dev(G, dt), empty_dev(x.shape, dt)
    adam = adam_struct()
    try:
        for bad in (-1, 2):
            with pytest.raises(B.LgaError) as e:
                st.forward_layer(bad, xd.data_ptr(), out.data_ptr())
            assert e.value.code == B.LGA_ERR_ARG
        with pytest.raises(B.LgaError) as e:
            st.backward_layer(0, Gd.data_ptr(), out.data_ptr(), None)           # no forward yet
        assert e.value.code == B.LGA_ERR_STATE
        with pytest.raises(B.LgaError) as e:
            st.forward_layer(0, None, out.data_ptr())
        assert e.value.code == B.LGA_ERR_ARG
        st.forward_layer(0, xd.data_ptr(), out.data_ptr())
        with pytest.raises(B.LgaError) as e:
            st.backward_layer(1, Gd.data_ptr(), out.data_ptr(), None)           # layer 1 has seen no input
        assert e.value.code == B.LGA_ERR_STATE
        with pytest.raises(B.LgaError) as e:
            st.backward_layered(Gd.data_ptr(), None, adam)                      # nor has the whole stack
        assert e.value.code == B.LGA_ERR_STATE
        st.backward_layer(0, Gd.data_ptr(), out.data_ptr(), adam)
        with pytest.raises(B.LgaError) as e:
            st.backward_layer(0, Gd.data_ptr(), out.data_ptr(), adam)           # weights changed since the forward
        assert e.value.code == B.LGA_ERR_STATE
        # forward into the next boundary, then layer 1 straight from that boundary, then the whole backward sweep
        st.forward_layer(0, xd.data_ptr(), None)
        st.forward_layer(1, st.checkpoint(1)[0], None)
        st.backward_layered(Gd.data_ptr(), out.data_ptr(), adam)
        torch.cuda.synchronize()
        assert torch.isfinite(out.float()).all()
    finally:
        st.close()
