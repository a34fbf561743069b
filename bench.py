#!/usr/bin/env python3
"""Benchmark of the layered-gradient-accumulation training step on one MI355X.

A step = lga_forward_layered + lga_backward_layered with fused per-layer Adam over one batch of
synthetic input (all n_mu micro-batches through all layers).  Inputs are resident in HBM before
the timed region.  Prints ONE JSON line:
  metric/value/unit  tokens per second of the whole step
  roofline           the dominant kernel's achieved rate against the MI355X peak, from HIP event
                     pairs the library records around every launch inside the timed region
  cpu_baseline       the fp64 numpy oracle timed on the host cores on a bounded sample
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3       # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E

DEFAULT_GROUP = {0: 4, 1: 4, 2: 4, 3: 4, 4: 4}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="index into the five benchmark configurations")
    ap.add_argument("--x-family", type=int, default=0, metavar="X",
                    help="instead of --config: the paper's X_[x] model (table B.1), all x layers, micro-batches of one "
                         "sequence; --n-micro sets how many")
    ap.add_argument("--layers", type=int, default=0,
                    help="with --x-family: run this many of the model's layers (0 = all x of them)")
    ap.add_argument("--heads", type=int, default=0,
                    help="override the configuration's number of heads (cfg4 with 80 heads is X_160's own 320-wide head)")
    ap.add_argument("--n-micro", type=int, default=0,
                    help="micro-batches per step: of the --x-family workload (default 32), or instead of the benchmark "
                         "configuration's own (for traffic-versus-n measurements; the workload name then says so)")
    ap.add_argument("--attention", choices=["causal", "full"], default="causal",
                    help="full: the paper's encoder, no mask (the benchmark configurations are causal decoders)")
    ap.add_argument("--group", type=int, default=0, help="micro-batches per kernel launch (0 = default for the config)")
    ap.add_argument("--order", choices=["layered", "mbmajor"], default="layered")
    ap.add_argument("--overlap", type=int, default=0, choices=[0, 1, 2, 3],
                    help="bits: 1 = restores, 2 = per-layer Adam steps on the library's second stream beside the layer sweeps")
    ap.add_argument("--param-buffers", type=int, default=0,
                    help="16-bit parameter buffers kept (0 = one per layer); fewer makes the orders differ in restore traffic")
    ap.add_argument("--offload", action="store_true",
                    help="keep the layer-boundary activations in pinned host memory (two slots on the device)")
    ap.add_argument("--fp16", action="store_true",
                    help="run the 16-bit configuration in IEEE half instead of bfloat16, with the per-layer non-finite "
                         "test before each Adam step (not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=64)
    ap.add_argument("--kernels", action="store_true", help="also print the per-kernel table to stderr")
    return ap.parse_args()


def measured_traffic(workload, kernel):
    """HBM-side bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this
    workload (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy of known size), or None."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.rstrip("\n").split("\t")
                if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel:
                    return float(parts[2])
    except OSError:
        pass
    return None


def cpu_baseline(w, sample_tokens, causal=True):
    """Time the oracle (as it stands) on a one-layer, one-micro-batch sample of the same layer shape."""
    import numpy as np
    import synth_inputs as S
    from oracle import lga_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    s = min(w.seq_len, sample_tokens)
    sw = S.Workload(w.name + "_cpu_sample", 1, w.d_model, w.n_heads, w.d_ff, s, 1, 1, w.dtype)
    x, G, params = S.make_inputs(sw, seed=0)
    shape = O.StackShape(d_l=1, d_m=sw.d_model, d_a=sw.n_heads, d_I=sw.d_ff, d_s=s, b_mu=1, n_mu=1, causal=causal)
    t0 = time.perf_counter()
    O.step_microbatch_major(x, G, params, shape, O.AdamHyper())
    dt = time.perf_counter() - t0
    # the full workload does the same per-token work in each of its layers
    return {"value": s / dt / w.n_layers, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"fp64 numpy oracle, 1 layer x 1 micro-batch x {s} tokens of the same layer shape "
                      f"(d={w.d_model}, heads={w.n_heads}, d_ff={w.d_ff}), fwd+bwd+Adam in {dt:.2f} s; "
                      f"tokens/s scaled by 1/{w.n_layers} layers"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import synth_inputs as S
    from paper_2106_02679_amd import binding as B
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = S.x_family(args.x_family, args.n_micro or 32, n_layers=args.layers) if args.x_family else S.CONFIGS[args.config]
    if args.heads and args.heads != w.n_heads:
        w = S.Workload(f"{w.name}_h{args.heads}", w.n_layers, w.d_model, args.heads, w.d_ff, w.seq_len, w.micro_batch,
                       w.n_micro, w.dtype)
    if args.n_micro and not args.x_family and args.n_micro != w.n_micro:
        w = S.Workload(f"{w.name}_n{args.n_micro}", w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch,
                       args.n_micro, w.dtype)
    if args.fp16 and w.dtype == "bf16":
        w = S.Workload(w.name.replace("bf16", "fp16"), w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch,
                       w.n_micro, "fp16")
    dt = {"fp32": B.LGA_FP32, "bf16": B.LGA_BF16, "fp16": B.LGA_FP16}[w.dtype]
    is16 = dt != B.LGA_FP32
    # default group: the benchmark configurations' own, else about 4096 tokens per launch
    default_group = max(1, 4096 // (w.micro_batch * w.seq_len)) if args.x_family else DEFAULT_GROUP[args.config]
    group = args.group or default_group
    causal = args.attention == "causal"
    if args.order == "mbmajor":
        group = 1
    while w.n_micro % group:
        group -= 1
    cfg = B.make_config(w.n_layers, w.d_model, w.n_heads, w.d_ff, w.seq_len, w.micro_batch, w.n_micro, dt,
                        group=group, retain_grads=1 if args.order == "mbmajor" else 0, param_buffers=args.param_buffers,
                        overlap=args.overlap, attention=B.LGA_ATTN_CAUSAL if causal else B.LGA_ATTN_FULL,
                        offload_checkpoints=1 if args.offload else 0)
    torch.cuda.set_device(0)
    tdt = {B.LGA_FP32: torch.float32, B.LGA_BF16: torch.bfloat16, B.LGA_FP16: torch.float16}[dt]
    # half precision: every Adam step tests its layer's gradient first; the synthetic output gradient has unit variance,
    # thousands of times a real loss gradient, so it is its own "scaled" gradient (scale 1: nothing overflows, every
    # update is applied - "skipped_layer_updates" in the output line says so)
    loss_scale = 1.0 if dt == B.LGA_FP16 else 0.0
    shape = (w.n_micro, w.micro_batch, w.seq_len, w.d_model)
    gen = torch.Generator(device="cuda").manual_seed(0)
    x = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(tdt)
    dy = torch.randn(shape, device="cuda", dtype=torch.float32, generator=gen).to(tdt)      # "scaled" by loss_scale = 1
    st = B.Stack(cfg)                     # weights filled on the device: N(0, 0.02^2), gains 1, biases 0
    torch.cuda.synchronize()

    marks = []      # per timed step: events at its start, between the sweeps, at its end

    def step(t, timed=False):
        adam = B.lga_adam(1e-3, 0.9, 0.999, 1e-8, t, loss_scale, 1 if dt == B.LGA_FP16 else 0)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)] if timed else None
        if timed:
            ev[0].record()
        if args.order == "layered":
            st.forward_layered(x.data_ptr(), None)
            if timed:
                ev[1].record()
            st.backward_layered(dy.data_ptr(), None, adam)
        else:
            st.step_mbmajor(x.data_ptr(), dy.data_ptr(), None, None, adam)
            if timed:
                ev[1].record()
        if timed:
            ev[2].record()
            marks.append(ev)

    t = 1
    for _ in range(args.warmup):
        step(t); t += 1
    torch.cuda.synchronize()
    st.profile_begin()
    restores0 = st.restore_count()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        step(t, timed=True); t += 1
    e1.record()
    torch.cuda.synchronize()
    ms_total = e0.elapsed_time(e1)
    stats = st.profile_end()
    restores = (st.restore_count() - restores0) / args.steps
    skipped = sum(st.nonfinite_layers()) if dt == B.LGA_FP16 else 0       # layers whose last update was left out
    ms_step = ms_total / args.steps
    step_ms = [m[0].elapsed_time(m[2]) for m in marks]
    fwd_ms = [m[0].elapsed_time(m[1]) for m in marks]

    order = B.LGA_ORDER_LAYERED if args.order == "layered" else B.LGA_ORDER_MICROBATCH_MAJOR
    param_bytes, grad_bytes, flops_exec = B.traffic_model(cfg, order)
    P = w.params_per_layer
    tokens = w.tokens
    seqs = w.n_micro * w.micro_batch
    # the paper's count: 8 flop per token per parameter (appendix C.1) plus the attention products (2 forward,
    # 2 recompute, 5 backward; s^2 d flop each with the causal mask, twice that without)
    pair_factor = 1.0 if causal else 2.0
    flops_paper = 8.0 * tokens * P * w.n_layers + 9.0 * pair_factor * seqs * w.n_layers * w.seq_len ** 2 * w.d_model
    flops_model = 6.0 * tokens * P * w.n_layers + 7.0 * pair_factor * seqs * w.n_layers * w.seq_len ** 2 * w.d_model
    peak = PEAK_BF16_TFLOPS if is16 else PEAK_FP32_TFLOPS          # bf16 and fp16 MFMA: the same dense peak

    dom = stats[0]
    per_launch_ms = dom["ms"] / dom["launches"]
    is_hbm = dom["name"].startswith(("adam", "layernorm", "colsum", "cast"))
    if is_hbm:
        roof = {"bound": "hbm", "achieved": dom["bytes"] / dom["ms"] / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma" if is16 else "alu", "achieved": dom["flops"] / dom["ms"] / 1e9,
                "peak": peak, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    if roof["bound"] == "mfma":
        # calibration, measured live: what the chip sustains with nothing but MFMAs on register operands with random
        # mantissas and signs (its power management holds the clock below nominal on such data)
        import ctypes as C
        sink = torch.ones(65536 + (4 << 20) // 4, device="cuda")
        tf = C.c_double()
        B.check(B.lib.lga_op_mfma_rate(800000, 0, sink.data_ptr(), C.byref(tf), None))
        roof["mfma_only_rate_random_operands"] = tf.value
        roof["frac_of_mfma_only_rate"] = roof["achieved"] / tf.value
    roof["traffic"] = measured_traffic(w.name, dom["name"]) if (group == default_group and causal) else None
    roof["algorithmic_bytes_per_launch"] = dom["bytes"] / dom["launches"]
    roof["kernel"] = dom["name"]
    roof["launches"] = dom["launches"]
    roof["avg_launch_ms"] = per_launch_ms
    roof["share_of_step"] = dom["ms"] / ms_total

    gemm_ms = sum(k["ms"] for k in stats if k["name"].startswith("gemm"))
    gemm_fl = sum(k["flops"] for k in stats if k["name"].startswith("gemm"))
    out = {
        "metric": "tokens/sec fwd+bwd+Adam per GPT layer stack (1 GPU)",
        "value": tokens / (ms_step / 1e3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n_layers": w.n_layers, "d_model": w.d_model, "n_heads": w.n_heads,
                   "d_ff": w.d_ff, "seq_len": w.seq_len, "micro_batch": w.micro_batch, "n_micro": w.n_micro,
                   "group": group, "order": args.order, "attention": args.attention, "tokens_per_step": tokens,
                   "param_buffers": args.param_buffers or w.n_layers, "overlap": args.overlap,
                   "offload_checkpoints": bool(args.offload)},
        "ms_per_step_min": min(step_ms), "ms_per_step_max": max(step_ms),
        # layered order: forward sweep / backward sweep with recompute and the per-layer Adam steps (mean over the steps)
        "phase_ms": ({"forward": sum(fwd_ms) / len(fwd_ms), "backward_with_adam": ms_step - sum(fwd_ms) / len(fwd_ms),
                      "adam_kernels": sum(k["ms"] for k in stats if k["name"].startswith("adam")) / args.steps}
                     if args.order == "layered" else None),
        "restores_per_step": restores,
        "skipped_layer_updates": skipped,
        "device_arena_bytes": B.arena_bytes(cfg), "pinned_host_bytes": B.host_bytes(cfg),
        # checkpoint offload: every boundary goes to the host once, all but the top two come back once
        "pcie_bytes_per_step": (2 * w.n_layers * tokens * w.d_model * (2 if is16 else 4)) if args.offload else 0,
        "tflops_executed": flops_exec / ms_step / 1e9,
        "pct_peak_executed": 100.0 * flops_exec / ms_step / 1e9 / peak,
        "pct_peak_paper_flops": 100.0 * flops_paper / ms_step / 1e9 / peak,     # 8 p + 9 s^2 d accounting
        "pct_peak_model_flops": 100.0 * flops_model / ms_step / 1e9 / peak,     # 6 p + 7 s^2 d (no recompute)
        "all_gemm_tflops": gemm_fl / gemm_ms / 1e9 if gemm_ms > 0 else None,
        "all_gemm_share_of_step": gemm_ms / ms_total,
        "model_param_bytes_per_step": param_bytes, "model_grad_bytes_per_step": grad_bytes,
        "roofline": roof,
    }
    if args.kernels:
        for k in stats:
            print(f"{k['name']:<48} n={k['launches']:<6} ms={k['ms']:<10.3f} "
                  f"TFLOP/s={k['flops'] / k['ms'] / 1e9 if k['ms'] else 0:<8.1f} GB/s={k['bytes'] / k['ms'] / 1e6 if k['ms'] else 0:<8.1f}",
                  file=sys.stderr)
    st.close()
    del x, dy
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_tokens, causal)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
