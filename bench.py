#!/usr/bin/env python3
"""Benchmark of the layered-gradient-accumulation training step on one MI355X.

A step = lga_forward_layered + lga_backward_layered with fused per-layer Adam over one batch of
synthetic input (all n_mu micro-batches through all layers).  Inputs are resident in HBM before
the timed region.  Prints ONE JSON line:
  metric/value/unit  tokens per second of the whole step
  roofline           the dominant kernel's achieved rate against the MI355X peak, from HIP event
                     pairs the library records around every launch inside the timed region
  cpu_baseline       the fp64 numpy oracle timed on the host cores on a bounded sample
  audit              what the timed steps left behind (output, weights, gradient: finite? how large?), every step's
                     time, the dominant kernel's average per step, and the clock / power the board reported meanwhile

The timed steps are kept statistically alike: every step sees the same batch, so with the configurations' learning
rate of 1e-3 Adam would move every weight the same way step after step (its first steps are sign steps: 25 of them
shift each weight by more than the initial standard deviation of 0.02) and the operands of the later steps would no
longer be the workload's.  The benchmark therefore runs the same kernels with a learning rate of 1e-6 (`--lr`), which
leaves the weights within 0.2 % of their initial values over 25 steps; the arithmetic per step is identical, and the
audit reports the drift that did happen.
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
    ap.add_argument("--lr", type=float, default=1e-6,
                    help="Adam learning rate of the timed steps (see the module docstring; the parity tests use the "
                         "configurations' 1e-3 for their single step)")
    ap.add_argument("--no-audit", action="store_true", help="skip the read-back of output, weights and gradient")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-seq", type=int, default=256, help="positions per sequence of the oracle's sample")
    ap.add_argument("--cpu-sample-micro", type=int, default=2, help="micro-batches of the oracle's sample")
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


def cpu_baseline(w, n_micro, seq_len, causal=True):
    """Time the oracle (as it stands) on the workload's parity slice: one layer of the same shape (width, heads,
    feed-forward width), `n_micro` micro-batches of `seq_len` positions, forward + backward + Adam."""
    import numpy as np
    import synth_inputs as S
    from oracle import lga_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    s = min(w.seq_len, seq_len)
    n = min(w.n_micro, n_micro)
    sw = S.Workload(w.name + "_cpu_sample", 1, w.d_model, w.n_heads, w.d_ff, s, w.micro_batch, n, w.dtype)
    x, G, params = S.make_inputs(sw, seed=0)
    shape = O.StackShape(d_l=1, d_m=sw.d_model, d_a=sw.n_heads, d_I=sw.d_ff, d_s=s, b_mu=sw.micro_batch, n_mu=n, causal=causal)
    t0 = time.perf_counter()
    O.step_microbatch_major(x, G, params, shape, O.AdamHyper())
    dt = time.perf_counter() - t0
    # what the oracle multiplies: 2 flop per token and matrix entry forward, twice that backward (it stores instead of
    # recomputing); attention as full s x s products, 2 forward and 4 backward, 2 s^2 d flop each per sequence
    d, f = sw.d_model, sw.d_ff
    flops = 6.0 * sw.tokens * (4.0 * d * d + 2.0 * d * f) + 12.0 * n * sw.micro_batch * float(s) * s * d
    # the full workload does the same per-token work in each of its layers
    return {"value": sw.tokens / dt / w.n_layers, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "fp64_gflops": flops / dt / 1e9, "seconds": dt,
            "sample": f"fp64 numpy oracle on the workload's parity slice: 1 layer of the same shape (d={w.d_model}, "
                      f"heads={w.n_heads}, d_ff={w.d_ff}) x {n} micro-batches x {sw.micro_batch} x {s} positions = "
                      f"{sw.tokens} tokens, fwd+bwd+Adam in {dt:.1f} s (its per-parameter work - gradient buffers and "
                      f"Adam over {sw.params_per_layer / 1e9:.2f} G fp64 values - is included and does not shrink with "
                      f"the sample); tokens/s scaled by 1/{w.n_layers} layers"}


def gpu0_pci_address(torch):
    """'dddd:bb:dd.f' of cuda:0, or None where this torch does not report it."""
    try:
        p = torch.cuda.get_device_properties(0)
        return f"{p.pci_domain_id:04x}:{p.pci_bus_id:02x}:{p.pci_device_id:02x}.0"
    except Exception:
        return None


class BoardSampler:
    """Clock and power of GPU 0, sampled about once a second by a thread of its own while the timed steps run (host-side
    only, nothing is enqueued on the GPU).  Read from the driver's sysfs files of the device with GPU 0's PCI address;
    where those cannot be read, from `rocm-smi` in a child process - but not under a profiler, whose preloaded library
    would come up inside that child."""

    def __init__(self, period=1.0, pci=None):
        import glob
        import shutil
        import threading
        self.period = period
        self.samples = []           # (sclk MHz or None, W or None)
        self.sysfs = None
        if pci:
            for dev in glob.glob("/sys/class/drm/card*/device"):
                if os.path.realpath(dev).lower().endswith(pci.lower()) and os.access(os.path.join(dev, "pp_dpm_sclk"), os.R_OK):
                    self.sysfs = dev
        under_profiler = any("rocprof" in os.environ.get(k, "").lower() for k in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "HSA_TOOLS_LIB"))
        self.exe = None
        if not self.sysfs and not under_profiler:
            self.exe = shutil.which("rocm-smi") or ("/opt/rocm/bin/rocm-smi" if os.path.exists("/opt/rocm/bin/rocm-smi") else None)
        self._stop = threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True) if (self.sysfs or self.exe) else None

    def _once_sysfs(self):
        import glob
        import re
        sclk = pw = None
        try:
            cur = [l for l in open(os.path.join(self.sysfs, "pp_dpm_sclk")).read().splitlines() if l.rstrip().endswith("*")]
            m = re.search(r"(\d+)\s*mhz", cur[0].lower()) if cur else None
            sclk = int(m.group(1)) if m else None
        except OSError:
            pass
        for name in ("power1_average", "power1_input"):
            for f in glob.glob(os.path.join(self.sysfs, "hwmon", "hwmon*", name)):
                try:
                    pw = int(open(f).read().strip()) / 1e6          # microwatts
                except (OSError, ValueError):
                    continue
                break
            if pw is not None:
                break
        self.samples.append((sclk, pw))

    def _once(self):
        import re
        import subprocess
        if self.sysfs:
            return self._once_sysfs()
        try:
            txt = subprocess.run([self.exe, "-d", "0", "--showclocks", "--showpower"], capture_output=True, text=True,
                                 timeout=10).stdout
        except Exception:
            return
        sclk = re.search(r"sclk clock level[^(]*\((\d+)Mhz\)", txt)
        pw = re.search(r"Power[^:\n]*\(W\)\s*:\s*([0-9.]+)", txt)
        self.samples.append((int(sclk.group(1)) if sclk else None, float(pw.group(1)) if pw else None))

    def _run(self):
        while not self._stop.is_set():
            self._once()
            self._stop.wait(self.period)

    def start(self):
        if self._thread:
            self._thread.start()

    def stop(self):
        if not self._thread:
            return None
        self._stop.set()
        self._thread.join(timeout=15)
        clk = [c for c, _ in self.samples if c is not None]
        pw = [p for _, p in self.samples if p is not None]
        mean = lambda v: sum(v) / len(v) if v else None
        return {"samples": len(self.samples), "sclk_mhz_mean": mean(clk), "sclk_mhz_min": min(clk) if clk else None,
                "sclk_mhz_max": max(clk) if clk else None, "power_w_mean": mean(pw), "power_w_max": max(pw) if pw else None,
                "source": (f"sysfs {self.sysfs}: pp_dpm_sclk, hwmon power" if self.sysfs else "rocm-smi --showclocks --showpower")
                          + ", one sample per second during the timed steps"}


AUDIT_CHUNK = 1 << 28          # elements per piece of a read-back (at most 1 GiB of fp32 on the device at a time)


def tensor_audit(torch, B, ptr, count, tdt, keep=False, against=None):
    """finite? / rms / largest magnitude of `count` elements of type tdt at device (or pinned host) address ptr, read
    piece by piece.  keep: also return a device copy of the whole tensor; against: a tensor from an earlier call with
    keep - the relative change ||now - then|| / ||then|| is added to the result."""
    esz = torch.empty((), dtype=tdt).element_size()
    whole = torch.empty(count, device="cuda", dtype=tdt) if keep else None
    n_bad, sq, mx, num, den = 0, 0.0, 0.0, 0.0, 0.0
    for off in range(0, count, AUDIT_CHUNK):
        n = min(AUDIT_CHUNK, count - off)
        t = whole[off:off + n] if keep else torch.empty(n, device="cuda", dtype=tdt)
        B.copy_device(t.data_ptr(), ptr + off * esz, n * esz)
        torch.cuda.synchronize()
        n_bad += int(n - int(torch.isfinite(t).sum()))
        p = torch.nan_to_num(t.double(), nan=0.0, posinf=0.0, neginf=0.0)
        sq += float((p * p).sum())
        mx = max(mx, float(p.abs().max()))
        if against is not None:
            q = against[off:off + n].double()
            num += float((p - q).pow(2).sum())
            den += float((q * q).sum())
        del p, t
    out = {"all_finite": n_bad == 0, "nonfinite_count": n_bad, "rms": (sq / max(1, count)) ** 0.5, "abs_max": mx}
    if against is not None:
        out["relative_change"] = (num / den) ** 0.5 if den > 0 else None
    return out, whole


def profile_figures(workload, kernel):
    """avg launch duration (us) of `kernel` in the committed rocprofv3 --kernel-trace --stats summary of this workload,
    and the box-to-box spread that summary states, or (None, None)."""
    path = os.path.join(ROOT, "profiles", f"train_step_{workload}_kernel_stats.txt")
    avg = spread = None
    try:
        with open(path) as f:
            for line in f:
                parts = line.rstrip("\n").split("\t")
                if len(parts) == 3 and parts[0] == "rocprof_avg_us" and parts[1] == kernel:
                    avg = float(parts[2])
                if len(parts) == 2 and parts[0] == "box_to_box_spread":
                    spread = float(parts[1])
    except OSError:
        pass
    return avg, spread


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
    default_group = max(1, 4096 // (w.micro_batch * w.seq_len)) if args.x_family else S.BENCH_GROUP[args.config]
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
    audit = None
    if not args.no_audit:
        # layer 0's weights as initialised, kept (if they fit) to report how far the timed steps moved them
        ptr, n = st.params(0)
        free, _ = torch.cuda.mem_get_info()
        a0, w_start = tensor_audit(torch, B, ptr, n, torch.float32, keep=free > 4 * n + (24 << 30))
        audit = {"adam_lr": args.lr, "weights_layer0_start": a0}

    marks = []      # per timed step: events at its start, between the sweeps, at its end

    def step(t, timed=False):
        adam = B.lga_adam(args.lr, 0.9, 0.999, 1e-8, t, loss_scale, 1 if dt == B.LGA_FP16 else 0)
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

    # The last warm-up step is bracketed launch by launch: it names the dominant kernel and gives the per-kernel table.
    # The timed steps bracket that kernel alone (two event records per launch are a measurable share of a step of
    # thousands of short launches), unless --kernels asks for the table over the timed steps themselves.
    t = 1
    warm_stats = None
    for i in range(args.warmup):
        if i == args.warmup - 1:
            st.profile_begin()
        step(t); t += 1
        if i == args.warmup - 1:
            warm_stats = st.profile_end()
        print(f"[bench] warm-up step {i + 1}/{args.warmup} enqueued", file=sys.stderr, flush=True)
    torch.cuda.synchronize()
    only = None
    if warm_stats and not args.kernels:
        only = max(warm_stats, key=lambda k: k["ms"])["name"]
    restores0 = st.restore_count()
    sampler = BoardSampler(pci=gpu0_pci_address(torch))
    sampler.start()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    per_step_stats = []
    for _ in range(args.steps):
        # the library's per-launch event pairs are collected step by step (lga_profile_end waits for the step to
        # finish: one host round trip per step inside the timed region)
        st.profile_begin(only)
        step(t, timed=True); t += 1
        per_step_stats.append(st.profile_end())
        # one line per finished step on stderr: a run under a profiler or a watchdog shows that it is alive
        print(f"[bench] step {len(per_step_stats)}/{args.steps} done", file=sys.stderr, flush=True)
    e1.record()
    torch.cuda.synchronize()
    board = sampler.stop()
    ms_total = e0.elapsed_time(e1)
    merged = {}
    for one in per_step_stats:
        for k in one:
            m = merged.setdefault(k["name"], dict(name=k["name"], launches=0, ms=0.0, flops=0.0, bytes=0.0))
            for key in ("launches", "ms", "flops", "bytes"):
                m[key] += k[key]
    stats = sorted(merged.values(), key=lambda k: -k["ms"])
    # per-kernel table: over the timed steps if every launch was bracketed there, else the last warm-up step's
    table, table_steps = (stats, args.steps) if only is None else (warm_stats, 1)
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
        # calibration, measured live: what the chip sustains with nothing but MFMAs (in the GEMM loop's issue order) on
        # register operands with random mantissas and signs (its power management holds the clock below nominal on such data)
        import ctypes as C
        sink = torch.ones(65536, device="cuda")
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
    dom_per_step = [next((k["ms"] / k["launches"] for k in one if k["name"] == dom["name"]), None) for one in per_step_stats]
    roof["avg_launch_ms_per_step"] = dom_per_step
    # the committed rocprofv3 summary of this workload: its average for this kernel must agree with the live one
    prof_us, spread = profile_figures(w.name, dom["name"]) if (group == default_group and causal) else (None, None)
    if prof_us:
        live = per_launch_ms * 1e3
        roof["profile_avg_launch_us"] = prof_us
        roof["profile_frac"] = roof["frac"] * live / prof_us
        roof["live_over_profile"] = live / prof_us
        roof["agrees_with_profile"] = abs(live / prof_us - 1.0) <= (spread or 0.05)
        if not roof["agrees_with_profile"]:
            roof["note"] = (f"this run's average launch of {dom['name']} ({live:.0f} us) differs from the committed profile's "
                            f"({prof_us:.0f} us) by more than the stated box-to-box spread of {100 * (spread or 0.05):.0f} %: "
                            "frac is this run's, profile_frac the profile's")
    if audit is not None:
        ptr, nbytes = st.checkpoint(w.n_layers)
        audit["output_y"], _ = tensor_audit(torch, B, ptr, nbytes // (2 if is16 else 4), tdt)
        ptr, n = st.params(0)
        audit["weights_layer0_end"], _ = tensor_audit(torch, B, ptr, n, torch.float32, against=w_start)
        audit["weights_layer0_relative_change"] = audit["weights_layer0_end"].pop("relative_change", None)
        del w_start
        try:
            last = 0 if args.order == "layered" else w.n_layers - 1        # the layer whose gradient the buffer still holds
            ptr, n = st.grads(last)
            audit["gradient_last_layer_done"], _ = tensor_audit(torch, B, ptr, n, torch.float32)
        except B.LgaError:
            audit["gradient_last_layer_done"] = None
        audit["all_finite"] = all(v["all_finite"] for k, v in audit.items() if isinstance(v, dict) and "all_finite" in v)
        audit["board"] = board

    gemm_ms = sum(k["ms"] for k in table if k["name"].startswith("gemm")) / table_steps
    gemm_fl = sum(k["flops"] for k in table if k["name"].startswith("gemm")) / table_steps
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
                   "offload_checkpoints": bool(args.offload), "adam_lr": args.lr},
        "ms_per_step_min": min(step_ms), "ms_per_step_max": max(step_ms), "ms_per_step_list": step_ms,
        # layered order: forward sweep / backward sweep with recompute and the per-layer Adam steps (mean over the steps)
        "phase_ms": ({"forward": sum(fwd_ms) / len(fwd_ms), "backward_with_adam": ms_step - sum(fwd_ms) / len(fwd_ms),
                      "adam_kernels": sum(k["ms"] for k in table if k["name"].startswith("adam")) / table_steps}
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
        "all_gemm_share_of_step": gemm_ms / ms_step,
        "per_kernel_table_from": "timed steps" if only is None else "last warm-up step (timed steps bracket the dominant kernel only)",
        "model_param_bytes_per_step": param_bytes, "model_grad_bytes_per_step": grad_bytes,
        "roofline": roof,
        "audit": audit,
    }
    if args.kernels:
        for k in table:
            print(f"{k['name']:<48} n={k['launches']:<6} ms={k['ms']:<10.3f} "
                  f"TFLOP/s={k['flops'] / k['ms'] / 1e9 if k['ms'] else 0:<8.1f} GB/s={k['bytes'] / k['ms'] / 1e6 if k['ms'] else 0:<8.1f}",
                  file=sys.stderr)
    st.close()
    del x, dy
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_micro, args.cpu_sample_seq, causal)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
