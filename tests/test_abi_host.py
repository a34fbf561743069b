"""CPU-only checks of the boundary: the library loads, exports every symbol the headers declare,
and its host-side logic (validation, sizing, traffic model) behaves.  No kernel is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2106_02679_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(lga_\w+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"lga_init_stack", "lga_forward_layered", "lga_backward_layered", "lga_adam_step_layer", "lga_grads"} <= names
    for name in names:
        assert hasattr(B.lib, name), name
    assert names == set(B.SIGNATURES), names ^ set(B.SIGNATURES)


def cfg(**kw):
    base = dict(n_layers=2, d_model=64, n_heads=4, d_ff=256, seq_len=32, micro_batch=2, n_micro=4, dtype=B.LGA_FP32,
                group=1, retain_grads=0)
    base.update(kw)
    return B.make_config(**base)


def test_parameter_count_follows_table_b1_closed_form():
    # Table B.1: p = 12 x^5 + 13 x^3 with d_m = x^2, d_l = x  =>  p_l = 12 d_m^2 + 13 d_m ; X_2 has 488
    assert 2 * B.params_per_layer(cfg(d_model=4, n_heads=1, d_ff=16)) == 488
    for d in (64, 768, 12288, 25600):
        assert B.params_per_layer(cfg(d_model=d, n_heads=d // 64 if d > 64 else 4, d_ff=4 * d)) == 12 * d * d + 13 * d


@pytest.mark.parametrize("kw,code", [
    (dict(n_layers=0), B.LGA_ERR_SHAPE), (dict(d_model=65), B.LGA_ERR_SHAPE), (dict(group=3), B.LGA_ERR_SHAPE),
    (dict(group=0), B.LGA_ERR_SHAPE), (dict(group=8), B.LGA_ERR_SHAPE), (dict(dtype=7), B.LGA_ERR_ARG),
    (dict(dtype=B.LGA_BF16, d_model=48, d_ff=192), B.LGA_ERR_SHAPE),    # d_h = 12 is not a multiple of 8
    # d_h = 256 > 160 has no fused attention kernel, and 8196 is not a multiple of 8, which the GEMM-built attention
    # needs: the one-wavefront kernels remain, whose LDS rows end below this length
    (dict(dtype=B.LGA_BF16, d_model=1024, d_ff=4096, seq_len=8196), B.LGA_ERR_SHAPE),
    (dict(attention=2), B.LGA_ERR_ARG), (dict(offload_checkpoints=2), B.LGA_ERR_ARG),
    (dict(dtype=B.LGA_BF16, d_model=128, n_heads=4, d_ff=500), B.LGA_ERR_SHAPE),
    (dict(seq_len=0), B.LGA_ERR_SHAPE),
    # leading dimensions of the 16-bit GEMM operands end at 2 097 151 elements: one group's tokens + 64 ...
    (dict(dtype=B.LGA_BF16, d_model=64, n_heads=4, d_ff=256, seq_len=2097088, micro_batch=1, n_micro=1), B.LGA_ERR_SHAPE),
    # ... and an explicit number of merged weight-gradient groups times that
    (dict(dtype=B.LGA_BF16, d_model=64, n_heads=4, d_ff=256, seq_len=1048576, micro_batch=1, n_micro=4, wgrad_groups=2),
     B.LGA_ERR_SHAPE),
])
def test_bad_configurations_are_refused_on_the_host(kw, code):
    out = C.c_uint64()
    assert B.lib.lga_arena_bytes(C.byref(cfg(**kw)), C.byref(out)) == code
    assert B.last_error()
    h = C.c_void_p()
    assert B.lib.lga_init_stack(C.byref(cfg(**kw)), None, C.byref(h)) == code
    assert not h.value


def test_automatic_merging_of_weight_gradient_gemms_respects_the_leading_dimension_limit():
    # 4 groups of 1 048 576 tokens: two of them side by side would need a row pitch of 2 097 216 > 2 097 151, so the
    # automatic choice must be 1 group per GEMM - the arena of the explicit setting
    # (64 layers: their checkpoints make the arena large enough that the memory rule alone would merge all four)
    long = dict(dtype=B.LGA_BF16, n_layers=64, d_model=64, n_heads=4, d_ff=256, seq_len=1048576, micro_batch=1, n_micro=4)
    assert B.arena_bytes(cfg(**long, wgrad_groups=0)) == B.arena_bytes(cfg(**long, wgrad_groups=1))
    # a quarter as long: all four groups fit one pitch, and the automatic choice merges them
    shorter = dict(long, seq_len=262144)
    assert B.arena_bytes(cfg(**shorter, wgrad_groups=0)) == B.arena_bytes(cfg(**shorter, wgrad_groups=4))


def test_large_heads_get_a_workspace_for_the_gemm_built_attention():
    # d_h = 256 (4 heads) against d_h = 128 (8 heads) at the same width: the arenas differ by the workspace - one
    # sequence's score matrices, 12 s^2 bytes per head, for as many heads as fit 4 GiB - less the four extra heads'
    # rows in the two softmax-statistics buffers (4 bytes per head, position and sequence of a group)
    wide = dict(dtype=B.LGA_BF16, d_model=1024, d_ff=4096)
    assert B.lib.lga_op_attention_gemm_workspace_bytes(1024, 4) == 12 * 1024 * 1024 * 4

    def extra(heads_in_workspace, **kw):
        c4, c8 = cfg(**wide, **kw), cfg(**wide, n_heads=8, **kw)
        stats = 2 * 4 * (8 - 4) * c4.group * c4.micro_batch * c4.seq_len
        return B.arena_bytes(c4) - B.arena_bytes(c8) + stats - 12 * c4.seq_len ** 2 * heads_in_workspace

    assert 0 <= extra(4, seq_len=1024) < 4096
    assert 0 <= extra(4, seq_len=8192) < 4096                                     # 3.2 GB: all four heads still fit
    assert 0 <= extra(1, seq_len=16384, micro_batch=1, n_micro=1) < 4096          # 3.2 GB per head: one at a time


def test_null_arguments():
    h = C.c_void_p()
    assert B.lib.lga_init_stack(None, None, C.byref(h)) == B.LGA_ERR_ARG
    assert B.lib.lga_init_stack(C.byref(cfg()), None, None) == B.LGA_ERR_ARG
    assert B.lib.lga_forward_layered(None, None, None) == B.LGA_ERR_ARG
    assert B.lib.lga_grads(None, 0, None, None) == B.LGA_ERR_ARG
    B.lib.lga_destroy_stack(None)      # must be a no-op


def test_arena_holds_state_checkpoints_and_scratch():
    c = cfg(n_layers=4, d_model=12288, n_heads=96, d_ff=49152, seq_len=2048, micro_batch=1, n_micro=32,
            dtype=B.LGA_BF16, group=2, retain_grads=0, wgrad_groups=1)
    P = 12 * 12288 ** 2 + 13 * 12288
    T = 32 * 2048
    state = 12 * 4 * P                              # appendix C.3: 12 p bytes of fp32 parameters and moments
    one_grad_buffer = 4 * P
    copies16 = 2 * 2 * 4 * P                        # 16-bit weights and their transposed copy
    ckpts = 2 * 5 * T * 12288 + 2 * T * 12288       # L+1 boundaries and the running activation gradient
    total = B.arena_bytes(c)
    assert total > state + one_grad_buffer + copies16 + ckpts
    assert total < 1.15 * (state + one_grad_buffer + copies16 + ckpts)      # scratch is a small addition
    assert total < 288e9
    # keeping every layer's gradient costs exactly (L-1) more buffers
    c2 = cfg(n_layers=4, d_model=12288, n_heads=96, d_ff=49152, seq_len=2048, micro_batch=1, n_micro=32,
             dtype=B.LGA_BF16, group=2, retain_grads=1, wgrad_groups=1)
    assert abs((B.arena_bytes(c2) - total) - 3 * 4 * P) < 4096
    # merging the weight-gradient GEMMs of w groups keeps w - 1 more groups of transposed operands:
    # 2 bytes x (2 d_ff + 8 d_model) rows x group tokens each
    c4 = cfg(n_layers=4, d_model=12288, n_heads=96, d_ff=49152, seq_len=2048, micro_batch=1, n_micro=32,
             dtype=B.LGA_BF16, group=2, retain_grads=0, wgrad_groups=4)
    per_group = 2 * (2 * 49152 + 8 * 12288) * (2 * 2048)
    assert abs((B.arena_bytes(c4) - total) - 3 * per_group) < 65536
    # automatic choice: bounded by a quarter of everything else, and never beyond the number of groups
    ca = cfg(n_layers=4, d_model=12288, n_heads=96, d_ff=49152, seq_len=2048, micro_batch=1, n_micro=32,
             dtype=B.LGA_BF16, group=2, retain_grads=0, wgrad_groups=0)
    auto = B.arena_bytes(ca)
    assert total <= auto <= 1.25 * total
    assert auto - total <= 15 * per_group + 65536
    assert B.lib.lga_arena_bytes(C.byref(cfg(wgrad_groups=5)), C.byref(C.c_uint64())) == B.LGA_ERR_SHAPE   # > n_micro / group


def test_traffic_model_layered_is_independent_of_micro_batch_count_when_fully_grouped():
    def model(n, g, order):
        c = cfg(n_layers=1, d_model=1024, n_heads=8, d_ff=4096, seq_len=128, micro_batch=1, n_micro=n,
                dtype=B.LGA_BF16, group=g, retain_grads=1)
        return B.traffic_model(c, order)
    p8, g8, f8 = model(8, 8, B.LGA_ORDER_LAYERED)
    p32, g32, f32_ = model(32, 32, B.LGA_ORDER_LAYERED)
    assert p8 == p32 and g8 == g32                    # bytes do not grow with n
    assert abs(f32_ / f8 - 4.0) < 1e-12               # flops do
    pm, gm, fm = model(32, 1, B.LGA_ORDER_MICROBATCH_MAJOR)
    P = 12 * 1024 ** 2 + 13 * 1024
    Pm = 12 * 1024 ** 2
    assert gm == 8 * P + 31 * 8 * P                   # first write + Adam read, then read-modify-write per micro-batch
    assert g32 == 8 * P
    # layered, 8 groups of 4: vectors are read-modify-written per group, matrices once per merged GEMM
    def grads(w):
        c = cfg(n_layers=1, d_model=1024, n_heads=8, d_ff=4096, seq_len=128, micro_batch=1, n_micro=32,
                dtype=B.LGA_BF16, group=4, retain_grads=0, wgrad_groups=w)
        return B.traffic_model(c, B.LGA_ORDER_LAYERED)[1]
    assert grads(1) == 8 * P + 7 * 8 * P
    assert grads(4) == 8 * P + 7 * 8 * (P - Pm) + 1 * 8 * Pm
    assert grads(8) == 8 * P + 7 * 8 * (P - Pm)
    assert pm - p32 == 31 * 2 * (3 * Pm - 1024 * 4096)
    assert fm == f32_


def test_traffic_model_restores_are_constant_in_n_when_layered_and_proportional_otherwise():
    """Figure 2 / table C.1 with two parameter buffers for a deeper stack: the layered order restores each layer
    about once per pass whatever the number of micro-batches; the micro-batch-major order once per pass and
    micro-batch."""
    L, d, f = 6, 1024, 4096
    P, Pm = 12 * d * d + 13 * d, 12 * d * d
    restore = 4 * P + 2 * P + 4 * Pm                   # read masters, write the 16-bit copy, re-read / write its transpose

    def extra(n, order, buffers):
        kw = dict(n_layers=L, d_model=d, n_heads=8, d_ff=f, seq_len=128, micro_batch=1, n_micro=n, dtype=B.LGA_BF16,
                  group=1, retain_grads=1)
        full = B.traffic_model(cfg(param_buffers=0, **kw), order)[0]
        return B.traffic_model(cfg(param_buffers=buffers, **kw), order)[0] - full

    # layered, 2 buffers, 6 layers: forward restores layers 2..5 (0, 1 are left from the previous backward), backward 3..0
    assert extra(8, B.LGA_ORDER_LAYERED, 2) == 8 * restore
    assert extra(64, B.LGA_ORDER_LAYERED, 2) == 8 * restore
    # micro-batch-major: the same 8 for every micro-batch (each ends with layers 1 and 0 resident); Adam at the
    # end of the step refreshes only those two layers' copies
    for n in (8, 64):
        assert extra(n, B.LGA_ORDER_MICROBATCH_MAJOR, 2) == 8 * n * restore - (L - 2) * (2 * P + 4 * Pm)
    assert extra(8, B.LGA_ORDER_LAYERED, L) == 0
    assert B.lib.lga_arena_bytes(C.byref(cfg(param_buffers=3)), C.byref(C.c_uint64())) == B.LGA_ERR_SHAPE   # > n_layers
    # the arena shrinks by the copies of the layers that are no longer resident
    kw = dict(n_layers=L, d_model=d, n_heads=8, d_ff=f, seq_len=128, micro_batch=1, n_micro=8, dtype=B.LGA_BF16)
    assert abs((B.arena_bytes(cfg(**kw)) - B.arena_bytes(cfg(param_buffers=2, **kw))) - (L - 2) * 4 * P) < 4096


def test_flop_model_against_the_papers_count():
    # Appendix C.1: 8 flop per token per parameter with full recompute.  The library skips the second
    # feed-forward GEMM in recompute (its output is not needed), i.e. executes 8 - 2 * (d d_I / p_matrices).
    c = cfg(n_layers=3, d_model=1024, n_heads=8, d_ff=4096, seq_len=64, micro_batch=2, n_micro=4, dtype=B.LGA_BF16)
    _, _, flops = B.traffic_model(c, B.LGA_ORDER_LAYERED)
    tokens, Pm = 4 * 2 * 64, 12 * 1024 ** 2
    gemm = 2.0 * tokens * 3 * (4 * Pm - 1024 * 4096)
    attn = 11.0 * (4 * 2) * 3 * 64 * 64 * 1024
    assert abs(flops - (gemm + attn)) / flops < 1e-12
    assert abs(gemm / (8.0 * tokens * 3 * Pm) - (1 - 1 / 12)) < 1e-12


def test_flop_model_doubles_the_attention_products_without_the_causal_mask():
    kw = dict(n_layers=3, d_model=1024, n_heads=8, d_ff=4096, seq_len=64, micro_batch=2, n_micro=4, dtype=B.LGA_BF16)
    _, _, causal = B.traffic_model(cfg(**kw), B.LGA_ORDER_LAYERED)
    _, _, full = B.traffic_model(cfg(attention=B.LGA_ATTN_FULL, **kw), B.LGA_ORDER_LAYERED)
    assert abs((full - causal) - 11.0 * (4 * 2) * 3 * 64 * 64 * 1024) / full < 1e-12


def test_checkpoint_offload_moves_the_boundaries_to_pinned_host_memory():
    kw = dict(n_layers=4, d_model=12288, n_heads=96, d_ff=49152, seq_len=2048, micro_batch=1, n_micro=32,
              dtype=B.LGA_BF16, group=4)
    boundary = 32 * 2048 * 12288 * 2
    assert B.host_bytes(cfg(**kw)) == 0
    assert B.host_bytes(cfg(offload_checkpoints=1, **kw)) == 5 * boundary
    # the device keeps two slots instead of L + 1 boundaries
    assert abs((B.arena_bytes(cfg(**kw)) - B.arena_bytes(cfg(offload_checkpoints=1, **kw))) - 3 * boundary) < 4096
    one = dict(kw, n_layers=1)
    assert B.arena_bytes(cfg(**one)) == B.arena_bytes(cfg(offload_checkpoints=1, **one))
    assert B.lib.lga_host_bytes(C.byref(cfg(**kw)), None) == B.LGA_ERR_ARG


def test_loss_scaler_matches_the_oracle_on_a_random_overflow_pattern():
    import numpy as np
    from oracle import lga_oracle as O
    rng = np.random.default_rng(7)
    c = B.lga_loss_scaler(65536.0, 2.0, 0.5, 1.0, 2.0 ** 24, 5, 0)
    o = O.LossScaler(scale=65536.0, growth=2.0, backoff=0.5, min_scale=1.0, max_scale=2.0 ** 24, growth_interval=5)
    for i in range(400):
        ov = bool(rng.random() < (0.5 if 100 <= i < 160 else 0.05))
        B.check(B.lib.lga_loss_scaler_update(C.byref(c), int(ov)))
        O.loss_scaler_update(o, ov)
        assert c.scale == o.scale and c.good_steps == o.good_steps, i
    assert 1.0 <= c.scale <= 2.0 ** 24
    for bad in (dict(scale=0.0), dict(growth=0.5), dict(backoff=0.0), dict(backoff=1.5), dict(growth_interval=0),
                dict(min_scale=0.0), dict(max_scale=0.5)):
        kw = dict(scale=8.0, growth=2.0, backoff=0.5, min_scale=1.0, max_scale=1024.0, growth_interval=2, good_steps=0)
        kw.update(bad)
        sc = B.lga_loss_scaler(**kw)
        assert B.lib.lga_loss_scaler_update(C.byref(sc), 0) == B.LGA_ERR_ARG, bad
    assert B.lib.lga_loss_scaler_update(None, 0) == B.LGA_ERR_ARG


def test_half_precision_mode_is_sized_like_bf16_and_follows_the_same_shape_rules():
    a = B.arena_bytes(cfg(dtype=B.LGA_BF16, seq_len=64))
    b = B.arena_bytes(cfg(dtype=B.LGA_FP16, seq_len=64))
    assert a == b
    assert B.traffic_model(cfg(dtype=B.LGA_FP16, seq_len=64), B.LGA_ORDER_LAYERED) == \
        B.traffic_model(cfg(dtype=B.LGA_BF16, seq_len=64), B.LGA_ORDER_LAYERED)
    out = C.c_uint64()
    assert B.lib.lga_arena_bytes(C.byref(cfg(dtype=B.LGA_FP16, d_model=60, n_heads=4)), C.byref(out)) == B.LGA_ERR_SHAPE
    assert B.lib.lga_arena_bytes(C.byref(cfg(dtype=3)), C.byref(out)) == B.LGA_ERR_ARG


def test_init_without_a_gpu_reports_a_hip_error_instead_of_crashing():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    h = C.c_void_p()
    assert B.lib.lga_init_stack(C.byref(cfg()), None, C.byref(h)) == B.LGA_ERR_HIP
    # the first HIP call of lga_init_stack (raising the large kernels' dynamic LDS limit) is the one that fails
    assert "dynamic LDS limit" in B.last_error() or "hipMalloc" in B.last_error()


@pytest.mark.parametrize("source,min_mfmas", [("gemm_bf16.hip", 12 * 128), ("mfma_rate.hip", 64)])
def test_generated_code_keeps_a_wait_state_between_two_mfmas_on_one_accumulator(tmp_path, source, min_mfmas):
    """The direct-to-LDS GEMM (and the MFMA-only calibration, which copies its issue order) issues a block's two
    products of a k tile back to back on the same accumulator through assembly statements the compiler does not model
    as matrix instructions; the hardware needs one wait state between the two.  The compiler's hazard pass supplies it:
    this test reads the device assembly it generates and fails if a toolchain ever stops doing so.  (Also: every
    accumulator update of that instruction is in place.)"""
    import shutil
    import subprocess
    from paper_2106_02679_amd import build as bld
    hipcc = bld._hipcc()
    if shutil.which(hipcc) is None and not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    asm = tmp_path / "device.s"
    flags = [f for f in bld.FLAGS if f not in ("-fPIC", "-Wall", "-Wno-unused-function")]
    res = subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", os.path.join(bld.CSRC, source), "-o", str(asm)],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    pat = re.compile(r"v_mfma_f32_16x16x32_\w+ (a\[\d+:\d+\]), v\[\d+:\d+\], v\[\d+:\d+\], (a\[\d+:\d+\])")
    n = pairs = 0
    last_dst, between = None, 0
    for line in asm.read_text().splitlines():
        t = line.strip()
        if not t or t.startswith(";") or (t.startswith(".") and not t.endswith(":")):
            continue
        m = pat.match(t)
        if m:
            n += 1
            assert m.group(1) == m.group(2), t                   # accumulates in place
            if m.group(1) == last_dst:
                pairs += 1
                assert between >= 1, f"no wait state before: {t}"
            last_dst, between = m.group(1), 0
        elif t.endswith(":"):
            last_dst = None                                       # a label: another path may arrive here
        else:
            between += 1
    assert n >= min_mfmas and pairs >= n // 4, (n, pairs)        # at least the unrolled loop of every kernel instance


def test_mfma_calibration_refuses_bad_arguments_before_touching_the_gpu():
    tf = C.c_double()
    sink = (C.c_float * 4)()
    for iters, mode, s, t in ((0, 0, sink, C.byref(tf)), ((1 << 23) + 1, 0, sink, C.byref(tf)), (10, 2, sink, C.byref(tf)),
                              (10, 0, None, C.byref(tf)), (10, 0, sink, None)):
        assert B.lib.lga_op_mfma_rate(iters, mode, s, t, None) == B.LGA_ERR_ARG
