"""Plumbing shared by the GPU parity tests: move seeded inputs to the device, run the C-ABI
library through its binding, bring results back as float64 numpy arrays."""
from __future__ import annotations

import numpy as np
import torch

import synth_inputs as S
from oracle import lga_oracle as O
from paper_2106_02679_amd import binding as B


TORCH_DTYPE = {B.LGA_FP32: torch.float32, B.LGA_BF16: torch.bfloat16, B.LGA_FP16: torch.float16}
DTYPE_CODE = {"fp32": B.LGA_FP32, "bf16": B.LGA_BF16, "fp16": B.LGA_FP16}
DTYPE_NAME = {v: k for k, v in DTYPE_CODE.items()}


def to_dev(a: np.ndarray, dtype: int) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(TORCH_DTYPE[dtype])


def empty_dev(shape, dtype: int) -> torch.Tensor:
    return torch.empty(shape, device="cuda", dtype=TORCH_DTYPE[dtype])


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def rel_err(a: np.ndarray, ref: np.ndarray) -> float:
    """Relative Frobenius error ||a - ref|| / ||ref|| (absolute norm if ref is all zero)."""
    a = np.asarray(a, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((a - ref).ravel())
    return float(num / den) if den > 0 else float(num)


def updatable_mask(w: S.Workload) -> np.ndarray:
    """Entries of a layer's flat parameter vector whose Adam update is well defined: everything but
    the key third of b_qkv, whose gradient is identically zero (softmax ignores a per-row score shift),
    so that its first-step update lr*g/(|g|+eps) is +-lr times the sign of rounding noise."""
    sl = S.tensor_slices(w.d_model, w.d_ff)
    keep = np.ones(w.params_per_layer, dtype=bool)
    keep[sl["b_qkv"].start + w.d_model: sl["b_qkv"].start + 2 * w.d_model] = False
    return keep


def dtype_code(w: S.Workload) -> int:
    return DTYPE_CODE[w.dtype]


def oracle_shape(w: S.Workload, causal: bool = True) -> O.StackShape:
    return O.StackShape(d_l=w.n_layers, d_m=w.d_model, d_a=w.n_heads, d_I=w.d_ff, d_s=w.seq_len,
                        b_mu=w.micro_batch, n_mu=w.n_micro, causal=causal)


def adam_struct(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, step=1, loss_scale=0.0, skip_nonfinite=0) -> B.lga_adam:
    return B.lga_adam(lr, beta1, beta2, eps, step, loss_scale, skip_nonfinite)


def adam_at_step(a: B.lga_adam, step: int) -> B.lga_adam:
    return B.lga_adam(a.lr, a.beta1, a.beta2, a.eps, step, a.loss_scale, a.skip_nonfinite)


def oracle_adam(a: B.lga_adam) -> O.AdamHyper:
    """The oracle gets the hyper-parameters as they cross the ABI: rounded to float32."""
    return O.AdamHyper(lr=float(np.float32(a.lr)), beta1=float(np.float32(a.beta1)), beta2=float(np.float32(a.beta2)),
                       eps=float(np.float32(a.eps)), step=int(a.step),
                       loss_scale=float(np.float32(a.loss_scale)) or 1.0, skip_nonfinite=bool(a.skip_nonfinite))


def compare_with_oracle(w, got, ref, gate, adam, zero_init=True):
    sl = S.tensor_slices(w.d_model, w.d_ff)
    d = w.d_model
    k_bias = slice(sl["b_qkv"].start + d, sl["b_qkv"].start + 2 * d)
    keep = np.ones(w.params_per_layer, dtype=bool)
    keep[k_bias] = False
    worst = {}
    for bnd in range(w.n_layers + 1):
        worst[f"act{bnd}"] = rel_err(got["boundaries"][bnd], ref.boundaries[bnd])
    worst["y"] = rel_err(got["y"], ref.boundaries[-1])
    worst["dx"] = rel_err(got["dx"], ref.dx)
    for l in range(w.n_layers):
        if got["grads"][l] is None:
            continue
        for name in S.PARAM_ORDER:
            worst[f"g{l}.{name}"] = rel_err(got["grads"][l][sl[name]], ref.grads[l][sl[name]])
        q_bias = slice(sl["b_qkv"].start, sl["b_qkv"].start + d)
        if w.dtype == "fp32":
            assert np.linalg.norm(got["grads"][l][k_bias]) <= 1e-4 * np.linalg.norm(got["grads"][l][q_bias])
        assert np.linalg.norm(ref.grads[l][k_bias]) <= 1e-12 * np.linalg.norm(ref.grads[l][q_bias])
    if adam is not None:
        for l in range(w.n_layers):
            worst[f"w{l}"] = rel_err(got["params"][l][keep], ref.new_params[l][keep])
            worst[f"m{l}"] = rel_err(got["m"][l], ref.new_m[l])
            # v is quadratic in the gradient, so a relative gradient error e shows up as 2e: gate at twice the gate
            worst[f"v{l}(halved)"] = 0.5 * rel_err(got["v"][l], ref.new_v[l])
            for name in S.PARAM_ORDER:
                if zero_init and name not in S.MATRICES and name not in S.GAINS:
                    continue
                sel = np.zeros(w.params_per_layer, dtype=bool)
                sel[sl[name]] = True
                sel &= keep
                worst[f"w{l}.{name}"] = rel_err(got["params"][l][sel], ref.new_params[l][sel])
    bad = {k: v for k, v in worst.items() if not v < gate}
    assert not bad, f"over the {gate} gate: {bad}; worst overall {max(worst.values()):.3e}"
    return worst


def run_gpu_step(w: S.Workload, x, G, params, *, group=1, retain=0, order="layered", adam=None, fused=True,
                 want_ckpt=True, wgrad_groups=0, param_buffers=0, overlap=0, attention=0,
                 offload=0, steps=1):
    """One training step through the C ABI.  Returns a dict of float64 numpy results."""
    dt = dtype_code(w)
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, dt,
                        group=group, retain_grads=retain, wgrad_groups=wgrad_groups, param_buffers=param_buffers,
                        overlap=overlap, attention=attention, offload_checkpoints=offload)
    st = B.Stack(cfg, np.concatenate(params))
    P = B.params_per_layer(cfg)
    xd, Gd = to_dev(x, dt), to_dev(G, dt)
    yd, dxd = empty_dev(x.shape, dt), empty_dev(x.shape, dt)
    out = {"grads": [None] * w.n_layers}
    np_dt = "float32"
    try:
        for extra in range(steps - 1):                    # earlier steps of a multi-step run (fused Adam, layered order)
            st.forward_layered(xd.data_ptr(), yd.data_ptr())
            st.backward_layered(Gd.data_ptr(), dxd.data_ptr(), adam_at_step(adam, adam.step + extra))
        if steps > 1:
            adam = adam_at_step(adam, adam.step + steps - 1)
        if order == "layered":
            st.forward_layered(xd.data_ptr(), yd.data_ptr())
            st.backward_layered(Gd.data_ptr(), dxd.data_ptr(), adam if (adam is not None and fused) else None)
        else:
            st.step_mbmajor(xd.data_ptr(), Gd.data_ptr(), yd.data_ptr(), dxd.data_ptr(), adam)
        torch.cuda.synchronize()
        for l in range(w.n_layers):
            try:
                ptr, n = st.grads(l)
                out["grads"][l] = B.read_device(ptr, n, np_dt).astype(np.float64)
            except B.LgaError:
                out["grads"][l] = None
        if adam is not None and order == "layered" and not fused:
            for l in range(w.n_layers):
                st.adam_step_layer(l, adam)
            torch.cuda.synchronize()
        out["y"] = to_host(yd)
        out["dx"] = to_host(dxd)
        if want_ckpt:
            n_act = int(np.prod(x.shape))
            ck = []
            for bnd in range(w.n_layers + 1):
                ptr, nbytes = st.checkpoint(bnd)
                if dt != B.LGA_FP32:
                    bits = B.read_device(ptr, n_act, "uint16")
                    ck.append(S.from_16bit_bits(bits, w.dtype).astype(np.float64).reshape(x.shape))
                else:
                    ck.append(B.read_device(ptr, n_act, "float32").astype(np.float64).reshape(x.shape))
            out["boundaries"] = np.stack(ck)
        out["params"], out["m"], out["v"] = [], [], []
        for l in range(w.n_layers):
            ptr, n = st.params(l)
            out["params"].append(B.read_device(ptr, n).astype(np.float64))
            mp, vp, n = st.moments(l)
            out["m"].append(B.read_device(mp, n).astype(np.float64))
            out["v"].append(B.read_device(vp, n).astype(np.float64))
        assert n == P
        out["restores"] = st.restore_count()
        if adam is not None and adam.skip_nonfinite:
            out["skipped"] = st.nonfinite_layers()
    finally:
        st.close()
    return out
