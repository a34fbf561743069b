"""GPU checks at the benchmark configurations' full sizes - cfg3, which bench.py times (4 layers, d = 12288,
96 heads, d_ff = 49152, seq 2048, 32 micro-batches), once more in IEEE half, and the two smaller bf16 configurations
cfg1 and cfg2 - in the launch configuration bench.py uses (layered order, group 4, single gradient buffer,
fused Adam, device-filled weights).

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
                                       B.LGA_BF16, group=4)) + 6 * w.tokens * w.d_model * 2 + 4e9
    if free < need:
        pytest.skip(f"needs about {need / 1e9:.0f} GB of free HBM")
    shape = (w.n_micro, w.micro_batch, w.seq_len, w.d_model)
    gen = torch.Generator(device="cuda").manual_seed(0)
    x = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(tdt)
    dy = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(tdt)
    a = _run(w, 4, x, dy, True)
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
    b = _run(w, 2, x, dy, False, offload=1)
    assert np.array_equal(a["y_head"], b["y_head"])
    for mu in a["samples"]:
        assert np.array_equal(a["samples"][mu], b["samples"][mu])
    for key in ("g_ln1", "g_bqkv", "g_wo_rows", "g_w2_rows"):
        assert rel_err(b[key], a[key]) < 1e-4, key
