"""Per-kernel benchmark of the layer stack's GEMM shapes and attention calls on one GPU.

    python -m paper_2106_02679_amd.opbench gemm      [--config 3] [--group 4] [--only NAME] [--iters 8]
    python -m paper_2106_02679_amd.opbench attention [--config 3] [--group 4] [--only fwd|bwd] [--iters 8] [--full]
    python -m paper_2106_02679_amd.opbench mfma      (the MFMA rate the chip sustains on register operands alone)

Every call goes through the C ABI's one-entry-point-per-kernel functions (lga_op_gemm, lga_op_attention_*),
on synthetic N(0, 1) activations and N(0, 0.02^2) weights of the benchmark configuration's shapes.  Times are
HIP-event averages over --iters launches after one warm-up launch.  Meant for profiling single kernels
(rocprofv3 --pmc ... -- python3 -m paper_2106_02679_amd.opbench ...); bench.py measures the whole step.
"""
import argparse
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def _time(fn, iters):
    import torch
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def gemm_shapes(w, group, wgrad_groups):
    """(name, epilogue, M, N, K) of every bf16 GEMM of one layer; all operands k-contiguous."""
    d, f = w.d_model, w.d_ff
    t = group * w.micro_batch * w.seq_len
    kw = wgrad_groups * t
    return [
        ("fwd qkv (bias)", 1, t, 3 * d, d), ("fwd out-proj (bias+resid)", 2, t, d, d),
        ("fwd ffn1 (bias+gelu)", 3, t, f, d), ("fwd ffn2 (bias+resid)", 2, t, d, f),
        ("dX ffn2 (x gelu')", 4, t, f, d), ("dX ffn1", 0, t, d, f), ("dX out-proj", 0, t, d, d), ("dX qkv", 0, t, d, 3 * d),
        ("dW ffn2 (fp32 out)", 5, f, d, kw), ("dW ffn1 (fp32 out)", 5, d, f, kw),
        ("dW out-proj (fp32 out)", 5, d, d, kw), ("dW qkv (fp32 out)", 5, d, 3 * d, kw),
    ]


def run_gemm(args):
    import torch
    import synth_inputs as S
    from paper_2106_02679_amd import binding as B
    w = S.CONFIGS[args.config]
    groups = w.n_micro // args.group
    bf = torch.bfloat16
    for name, epi, M, N, K in gemm_shapes(w, args.group, args.wgrad_groups or groups):
        if args.only and args.only not in name:
            continue
        # the stack's transposed weight-gradient operands have a row pitch of K + 64 elements: a power of two as pitch
        # sends the 256 rows of an operand tile to the same few memory channels (10 % slower at K = 65536)
        ld = K + 64 if epi == 5 else K
        A = torch.randn(M, ld, device="cuda", dtype=bf)
        Bm = (torch.randn(N, ld, device="cuda", dtype=torch.float32) * (1.0 if epi == 5 else 0.02)).to(bf)
        out = torch.empty(M, N, device="cuda", dtype=bf) if epi != 5 else None
        out2 = torch.empty(M, N, device="cuda", dtype=bf) if epi == 3 else None
        outf = torch.zeros(M, N, device="cuda", dtype=torch.float32) if epi == 5 else None
        bias = torch.zeros(N, device="cuda")
        aux = torch.randn(M, N, device="cuda", dtype=bf) if epi in (2, 4) else None
        ptr = lambda x: x.data_ptr() if x is not None else None

        slices = B.lib.lga_op_gemm_splitk_slices(M, N, K) if epi == 5 else 1
        scratch = torch.empty(slices * M * N, device="cuda") if slices > 1 else None

        def call():
            if epi == 5:      # the weight-gradient GEMM as the stack runs it (k range split when the output is small)
                B.check(B.lib.lga_op_gemm_splitk(B.LGA_BF16, M, N, K, A.data_ptr(), ld, Bm.data_ptr(), ld, outf.data_ptr(), N, 0.0,
                                                 ptr(scratch), slices * M * N, None))
            else:
                B.check(B.lib.lga_op_gemm(B.LGA_BF16, 1, 1, epi, M, N, K, A.data_ptr(), ld, Bm.data_ptr(), ld, ptr(out),
                                          ptr(out2), ptr(outf), N, bias.data_ptr(), ptr(aux), 0.0, None))
        ms = _time(call, args.iters)
        line = (f"{name:<28} M={M:<6} N={N:<6} K={K:<6} {ms:9.3f} ms {2.0 * M * N * K / ms / 1e9:8.1f} TFLOP/s"
                + (f"  ({slices} k slices)" if slices > 1 else ""))
        if args.library:
            # the plain product of the same operands into a 16-bit matrix (no epilogue; for the weight gradient the
            # library writes half the output bytes), best of three alternating rounds for both
            lib_out = torch.empty(M, N, device="cuda", dtype=bf)
            lib_call = lambda: torch.matmul(A[:, :K], Bm[:, :K].t(), out=lib_out)
            ours, theirs = [ms], []
            for _ in range(3):
                theirs.append(_time(lib_call, args.iters))
                ours.append(_time(call, args.iters))
            o, l = min(ours), min(theirs)
            line = (f"{name:<28} M={M:<6} N={N:<6} K={K:<6} {2.0 * M * N * K / o / 1e9:8.1f} TFLOP/s   vendor library "
                    f"{2.0 * M * N * K / l / 1e9:8.1f} TFLOP/s   ratio {l / o:.3f}")
            del lib_out
        print(line, flush=True)
        del A, Bm, out, out2, outf, aux, scratch
        torch.cuda.empty_cache()


def run_attention(args):
    import torch
    import synth_inputs as S
    from paper_2106_02679_amd import binding as B
    w = S.CONFIGS[args.config]
    n_seq, s, heads = args.group * w.micro_batch, w.seq_len, w.n_heads
    dh = w.d_model // heads
    d = heads * dh
    bf = torch.bfloat16
    qkv = torch.randn(n_seq * s, 3 * d, device="cuda", dtype=bf)
    dout = torch.randn(n_seq * s, d, device="cuda", dtype=bf)
    out = torch.empty(n_seq * s, d, device="cuda", dtype=bf)
    dqkv = torch.empty(n_seq * s, 3 * d, device="cuda", dtype=bf)
    lse = torch.empty(n_seq * heads * s, device="cuda")
    delta = torch.empty(n_seq * heads * s, device="cuda")

    def fwd():
        B.check(B.lib.lga_op_attention_fwd(B.LGA_BF16, 1, qkv.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, s, heads, dh, causal, None))

    def bwd():
        B.check(B.lib.lga_op_attention_bwd(B.LGA_BF16, 1, qkv.data_ptr(), out.data_ptr(), lse.data_ptr(), dout.data_ptr(),
                                           dqkv.data_ptr(), delta.data_ptr(), n_seq, s, heads, dh, causal, None))
    causal = 0 if args.full else 1
    pairs = n_seq * heads * s * s / (2.0 if causal else 1.0)            # visible (query, key) pairs
    fwd()
    for name, fn, flops in (("fwd", fwd, 4 * pairs * dh), ("bwd", bwd, 14 * pairs * dh)):
        if args.only and args.only != name:
            continue
        ms = _time(fn, args.iters)
        print(f"attention {name} n_seq={n_seq} s={s} heads={heads} d_h={dh}: {ms:8.3f} ms {flops / ms / 1e9:8.1f} TFLOP/s "
              f"({'causal' if causal else 'unmasked'}, executed flops)", flush=True)


def run_mfma(args):
    import ctypes as C
    import torch
    from paper_2106_02679_amd import binding as B
    sink = torch.zeros(65536, device="cuda")
    what = {1: "constant register operands", 0: "random register operands  "}
    for mode in (1, 0):
        for iters in (200000, 2000000):
            tf = C.c_double()
            B.check(B.lib.lga_op_mfma_rate(iters, mode, sink.data_ptr(), C.byref(tf), None))
            print(f"v_mfma_f32_16x16x32_bf16 only (two in a row per accumulator), {what[mode]}, {iters * 32} MFMAs per wavefront: {tf.value:8.1f} TFLOP/s",
                  flush=True)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("what", choices=["gemm", "attention", "mfma"])
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--group", type=int, default=4)
    ap.add_argument("--wgrad-groups", type=int, default=0, help="groups merged into one weight-gradient GEMM (0: all)")
    ap.add_argument("--only", default=None)
    ap.add_argument("--iters", type=int, default=8)
    ap.add_argument("--full", action="store_true", help="attention without the causal mask (encoder)")
    ap.add_argument("--library", action="store_true",
                    help="gemm: also time torch.matmul (the vendor library) on the same operands, alternating with this "
                         "library's kernel in the same process - context for the rates, never part of the product path")
    args = ap.parse_args()
    import torch
    assert torch.cuda.is_available(), "opbench needs a GPU"
    {"gemm": run_gemm, "attention": run_attention, "mfma": run_mfma}[args.what](args)


if __name__ == "__main__":
    main()
