"""GPU parity, kernel by kernel: each HIP kernel is called through the C ABI (lga_ops.h) on small,
ragged, multi-tile shapes and compared element-wise with the fp64 oracle's corresponding step.

Tolerances (relative Frobenius norm of the error):
  fp32 storage: 1e-5 (the gate the build is held to in fp32 mode).
  bf16 storage: inputs are bf16-exact and shared with the oracle, products accumulate in fp32, so the
  error is the rounding of the stored result, unit roundoff 2^-8 => about 2^-9/sqrt(3)*sqrt(2) ~ 1.6e-3
  rms per element; 4e-3 leaves a factor 2.5.  Attention rounds P (and dS) to bf16 before its second
  product, adding a similar term per product: 1e-2 forward, 2e-2 backward (the build's bf16 gate).
  fp16 storage (IEEE half): the same kernels with unit roundoff 2^-11, an eighth of bf16's: every 16-bit
  tolerance divided by 8 (5e-4; attention 1.25e-3 forward, 2.5e-3 backward).
"""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import lga_oracle as O
import synth_inputs as S
from paper_2106_02679_amd import binding as B
from gpu_helpers import to_dev, empty_dev, to_host, rel_err

F32, BF16, F16 = B.LGA_FP32, B.LGA_BF16, B.LGA_FP16
TOL_OUT = {F32: 1e-5, BF16: 4e-3, F16: 5e-4}
TOL_ATTN = {F32: (1e-5, 2e-5), BF16: (1e-2, 2e-2), F16: (1.25e-3, 2.5e-3)}
ROUND = {F32: lambda a: a, BF16: S.round_to_bf16, F16: S.round_to_fp16}


def rnd(rng, shape, dt, scale=1.0):
    a = (scale * rng.standard_normal(shape)).astype(np.float32)
    return ROUND[dt](a)


def with_half(cases):
    """The 16-bit cases of a list once more in IEEE half."""
    return cases + [(F16,) + c[1:] for c in cases if c[0] == BF16]


def fvec(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def gemm_oracle(A, Bm, akm, bkm):
    a = A if akm else A.T           # -> [M, K]
    b = Bm.T if bkm else Bm         # -> [K, N]
    return a.astype(np.float64) @ b.astype(np.float64)


GEMM_CASES = [
    # dtype, a_kmajor, b_kmajor, epilogue, M, N, K
    (F32, 1, 0, B.LGA_EPI_BIAS, 70, 45, 33),
    (F32, 1, 0, B.LGA_EPI_BIAS_RESID, 130, 64, 17),
    (F32, 1, 0, B.LGA_EPI_BIAS_GELU, 65, 129, 64),
    (F32, 1, 1, B.LGA_EPI_STORE, 67, 50, 40),
    (F32, 1, 1, B.LGA_EPI_MUL_DGELU, 64, 64, 70),
    (F32, 0, 0, B.LGA_EPI_ACCUM_F32, 45, 70, 100),
    (BF16, 1, 0, B.LGA_EPI_BIAS, 300, 392, 200),
    (BF16, 1, 0, B.LGA_EPI_STORE, 128, 128, 64),
    (BF16, 1, 0, B.LGA_EPI_BIAS_RESID, 257, 136, 72),
    (BF16, 1, 0, B.LGA_EPI_BIAS_GELU, 190, 264, 128),
    (BF16, 1, 1, B.LGA_EPI_STORE, 300, 200, 392),
    (BF16, 1, 1, B.LGA_EPI_MUL_DGELU, 131, 256, 136),
    (BF16, 1, 1, B.LGA_EPI_BIAS, 300, 392, 200),
    (BF16, 1, 1, B.LGA_EPI_BIAS_RESID, 257, 136, 72),
    (BF16, 1, 1, B.LGA_EPI_BIAS_GELU, 190, 264, 128),
    (BF16, 1, 1, B.LGA_EPI_ACCUM_F32, 200, 392, 304),
    (BF16, 1, 1, B.LGA_EPI_ACCUM_F32, 4104, 8200, 200),
    (BF16, 1, 1, B.LGA_EPI_BIAS_GELU, 4100, 8200, 136),
    (BF16, 0, 0, B.LGA_EPI_ACCUM_F32, 200, 392, 300),
    (BF16, 0, 0, B.LGA_EPI_STORE, 136, 72, 1000),
    # >= 512 tiles of 256x256: the large-tile kernel, with ragged edges in m, n and k
    (BF16, 1, 0, B.LGA_EPI_BIAS, 4100, 8200, 136),
    (BF16, 1, 1, B.LGA_EPI_STORE, 4100, 8200, 72),
    (BF16, 0, 0, B.LGA_EPI_ACCUM_F32, 4104, 8200, 200),
    # the large-tile kernel's row-store epilogues that read a second tensor, ragged in m and n
    (BF16, 1, 1, B.LGA_EPI_MUL_DGELU, 4100, 8200, 72),
    (BF16, 1, 1, B.LGA_EPI_BIAS_RESID, 4100, 8200, 72),
    (BF16, 1, 1, B.LGA_EPI_BIAS, 2050, 16392, 200),
    # tile grids that are whole 16 x 16 blocks of 256 x 256 tiles: the block-wise workgroup order
    (BF16, 1, 1, B.LGA_EPI_STORE, 4096, 4096, 72), (BF16, 1, 1, B.LGA_EPI_ACCUM_F32, 4096, 8192, 200),
    (BF16, 1, 1, B.LGA_EPI_BIAS_GELU, 8192, 4096, 136),
]


@pytest.mark.parametrize("case", with_half(GEMM_CASES), ids=lambda c: "-".join(map(str, c)))
def test_gemm_against_oracle_matmul(case):
    check_gemm(case)


# The large-tile kernel's k loop: a ring of five operand slots, a main loop unrolled over five k tiles that needs
# seven tiles ahead of it, a generic form for what is left, a tested form for the last two tiles and a prologue that
# has tile 1 in flight only if it exists.  Every k tile count from 1 to 13 (all residues of the ring, with and without
# the unrolled loop taking part), some with a ragged last tile, on the two workgroup orders.
K_SWEEP = [(BF16, 1, 1, (B.LGA_EPI_STORE, B.LGA_EPI_ACCUM_F32)[n % 2], 2048, 4096, 64 * n) for n in range(1, 14)] + \
          [(BF16, 1, 1, B.LGA_EPI_BIAS, 2048, 4096, K) for K in (328, 392, 456, 712, 776)] + \
          [(BF16, 1, 1, B.LGA_EPI_STORE, 4096, 4096, K) for K in (320, 448, 584)] + \
          [(F16, 1, 1, B.LGA_EPI_ACCUM_F32, 2048, 4096, K) for K in (384, 520)]


@pytest.mark.parametrize("case", K_SWEEP, ids=lambda c: "-".join(map(str, c)))
def test_large_tile_gemm_with_every_number_of_k_tiles(case):
    check_gemm(case)


def check_gemm(case):
    dt, akm, bkm, epi, M, N, K = case
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    pad = 8      # leading dimensions larger than the logical width: exercises pitches
    lda = (K if akm else M) + pad
    ldb = (K if bkm else N) + pad
    ldc = N + pad
    A = rnd(rng, (M if akm else K, lda), dt)
    Bm = rnd(rng, (N if bkm else K, ldb), dt)
    Al = A[:, :K] if akm else A[:, :M]
    Bl = Bm[:, :K] if bkm else Bm[:, :N]
    acc = gemm_oracle(Al, Bl, akm, bkm)
    bias = rng.standard_normal(N).astype(np.float32)
    aux = rnd(rng, (M, ldc), dt)
    old = rng.standard_normal((M, ldc)).astype(np.float32)
    beta = 1.0 if epi == B.LGA_EPI_ACCUM_F32 else 0.0
    Ad, Bd, auxd, biasd = to_dev(A, dt), to_dev(Bm, dt), to_dev(aux, dt), fvec(bias)
    out, out2 = empty_dev((M, ldc), dt), empty_dev((M, ldc), dt)
    out.zero_(); out2.zero_()
    outf = fvec(old)
    B.check(B.lib.lga_op_gemm(dt, akm, bkm, epi, M, N, K, Ad.data_ptr(), lda, Bd.data_ptr(), ldb, out.data_ptr(),
                              out2.data_ptr(), outf.data_ptr(), ldc, biasd.data_ptr(), auxd.data_ptr(), beta, None))
    torch.cuda.synchronize()
    a64 = aux[:, :N].astype(np.float64)
    tol = TOL_OUT[dt]
    if epi == B.LGA_EPI_STORE:
        assert rel_err(to_host(out)[:, :N], acc) < tol
    elif epi == B.LGA_EPI_BIAS:
        assert rel_err(to_host(out)[:, :N], acc + bias) < tol
    elif epi == B.LGA_EPI_BIAS_RESID:
        assert rel_err(to_host(out)[:, :N], acc + bias + a64) < tol
    elif epi == B.LGA_EPI_BIAS_GELU:
        u = acc + bias
        assert rel_err(to_host(out2)[:, :N], u) < tol
        assert rel_err(to_host(out)[:, :N], O.gelu(u)) < tol
    elif epi == B.LGA_EPI_MUL_DGELU:
        assert rel_err(to_host(out)[:, :N], acc * O.gelu_grad(a64)) < tol
    else:
        got = outf.cpu().numpy().astype(np.float64)
        assert rel_err(got[:, :N], old[:, :N].astype(np.float64) + acc) < 1e-5
        assert np.array_equal(got[:, N:], old[:, N:].astype(np.float64))      # padding untouched
        # beta = 0 must overwrite whatever was there (even NaN)
        outf.fill_(float("nan"))
        B.check(B.lib.lga_op_gemm(dt, akm, bkm, epi, M, N, K, Ad.data_ptr(), lda, Bd.data_ptr(), ldb, None, None,
                                  outf.data_ptr(), ldc, None, None, 0.0, None))
        torch.cuda.synchronize()
        assert rel_err(outf.cpu().numpy().astype(np.float64)[:, :N], acc) < 1e-5
    if epi != B.LGA_EPI_ACCUM_F32:
        assert np.all(to_host(out)[:, N:] == 0)                                # padding untouched


@pytest.mark.parametrize("dt,M,N,K,beta", [(BF16, 768, 768, 8192, 1.0), (BF16, 320, 264, 5000, 0.0),
                                           (BF16, 1032, 520, 40000, 1.0), (BF16, 256, 256, 1024 * 32 + 8, 0.0),
                                           (BF16, 768, 2304, 1000, 1.0), (F16, 768, 768, 8192, 1.0),
                                           (F16, 320, 264, 5000, 0.0)])
def test_weight_gradient_gemm_with_split_k_range(dt, M, N, K, beta):
    """Narrow outputs with a long contraction (the weight-gradient GEMMs of narrow layers): the k range is cut into
    slices that run as separate workgroups.  Against the fp64 product, against the unsplit kernel, twice (the
    scratch keeps the previous call's partial results), and bit-reproducibly; the last case is too short to split."""
    rng = np.random.default_rng(M + N + K)
    lda, ldb, ldc = K + 8, K + 16, N + 8
    A, Bm = rnd(rng, (M, lda), dt), rnd(rng, (N, ldb), dt)
    acc = A[:, :K].astype(np.float64) @ Bm[:, :K].astype(np.float64).T
    old = rng.standard_normal((M, ldc)).astype(np.float32)
    slices = B.lib.lga_op_gemm_splitk_slices(M, N, K)
    assert (slices > 1) == (K >= 2048)
    assert slices <= B.lib.lga_op_gemm_splitk_slices(M, N, 0)
    Ad, Bd = to_dev(A, dt), to_dev(Bm, dt)
    scratch = torch.full((slices * M * N,), float("nan"), device="cuda")
    ref = beta * old[:, :N].astype(np.float64) + acc
    results = []
    for attempt in range(2):
        outf = fvec(old)
        B.check(B.lib.lga_op_gemm_splitk(dt, M, N, K, Ad.data_ptr(), lda, Bd.data_ptr(), ldb, outf.data_ptr(), ldc, beta,
                                         scratch.data_ptr(), scratch.numel(), None))
        torch.cuda.synchronize()
        got = outf.cpu().numpy()
        assert rel_err(got[:, :N], ref) < 1e-5
        assert np.array_equal(got[:, N:], old[:, N:])                          # padding untouched
        results.append(got)
    assert np.array_equal(results[0], results[1])
    outf = fvec(old)
    B.check(B.lib.lga_op_gemm_splitk(dt, M, N, K, Ad.data_ptr(), lda, Bd.data_ptr(), ldb, outf.data_ptr(), ldc, beta, None, 0,
                                     None))                                    # no scratch: the unsplit kernel
    torch.cuda.synchronize()
    assert rel_err(outf.cpu().numpy()[:, :N], results[0][:, :N]) < 1e-5
    # scratch too small for the slices: falls back to the unsplit kernel instead of overrunning it
    if slices > 1:
        small = torch.zeros(M * N, device="cuda")
        outf = fvec(old)
        B.check(B.lib.lga_op_gemm_splitk(dt, M, N, K, Ad.data_ptr(), lda, Bd.data_ptr(), ldb, outf.data_ptr(), ldc, beta,
                                         small.data_ptr(), small.numel(), None))
        torch.cuda.synchronize()
        assert rel_err(outf.cpu().numpy()[:, :N], ref) < 1e-5


@pytest.mark.parametrize("R,C,pad", [(8, 8, 0), (136, 264, 8), (1000, 128, 0), (128, 3000, 16)])
def test_transpose(R, C, pad):
    rng = np.random.default_rng(R * C)
    a = rnd(rng, (R, C + pad), BF16)
    ad = to_dev(a, BF16)
    out = empty_dev((C, R + pad), BF16)
    out.zero_()
    B.check(B.lib.lga_op_transpose(ad.data_ptr(), out.data_ptr(), R, C, C + pad, R + pad, None))
    torch.cuda.synchronize()
    got = to_host(out)
    assert np.array_equal(got[:, :R], a[:, :C].T.astype(np.float64))
    assert np.all(got[:, R:] == 0)


@pytest.mark.parametrize("dt,R,C,pad", [(BF16, 8, 8, 0), (BF16, 136, 264, 8), (BF16, 1000, 128, 0), (F16, 128, 3000, 16),
                                         (F16, 4104, 776, 8), (BF16, 0, 64, 0)])
def test_transpose_that_also_returns_the_column_sums(dt, R, C, pad):
    """The transposing pass of the weight-gradient operands hands back the bias gradient (section 3: one gradient per
    layer, accumulated): the transposed matrix must be bit-exact, the sums those of the fp64 column sums, with beta 1
    and beta 0, on ragged tiles (R, C not multiples of 128) and padded leading dimensions."""
    rng = np.random.default_rng(R * C + 1)
    a = rnd(rng, (max(R, 1), C + pad), dt)[:R]
    ad = to_dev(a if R else np.zeros((1, C + pad), np.float32), dt)
    out = empty_dev((C, R + pad + (8 if R == 0 else 0)), dt)
    out.zero_()
    old = rng.standard_normal(C).astype(np.float32)
    sums = fvec(old)
    scratch = torch.empty(max(1, int(B.lib.lga_op_colsum_scratch_floats(R, C))), device="cuda")
    ldo = R + pad + (8 if R == 0 else 0)
    B.check(B.lib.lga_op_transpose_colsum(dt, ad.data_ptr(), out.data_ptr(), R, C, C + pad, ldo, 1.0, sums.data_ptr(),
                                          scratch.data_ptr(), None))
    torch.cuda.synchronize()
    got = to_host(out)
    assert np.array_equal(got[:, :R], a[:, :C].T.astype(np.float64))
    assert np.all(got[:, R:] == 0)
    ref = a[:, :C].astype(np.float64).sum(0)
    assert rel_err(sums.cpu().numpy(), old + ref) < 1e-5
    B.check(B.lib.lga_op_transpose_colsum(dt, ad.data_ptr(), out.data_ptr(), R, C, C + pad, ldo, 0.0, sums.data_ptr(),
                                          scratch.data_ptr(), None))
    torch.cuda.synchronize()
    if R:
        assert rel_err(sums.cpu().numpy(), ref) < 1e-5
    else:
        assert np.all(sums.cpu().numpy() == 0)
    assert B.lib.lga_op_transpose_colsum(F32, ad.data_ptr(), out.data_ptr(), R, C, C + pad, ldo, 0.0, sums.data_ptr(),
                                         scratch.data_ptr(), None) == B.LGA_ERR_ARG


def test_gemm_empty_and_rejected_arguments():
    t = torch.zeros(64, device="cuda")
    # M = 0: nothing to do, no launch
    B.check(B.lib.lga_op_gemm(F32, 1, 0, B.LGA_EPI_STORE, 0, 8, 8, t.data_ptr(), 8, t.data_ptr(), 8, t.data_ptr(), None,
                              None, 8, None, None, 0.0, None))
    # bf16 with N not a multiple of 8 is refused on the host
    rc = B.lib.lga_op_gemm(BF16, 1, 0, B.LGA_EPI_STORE, 8, 12, 8, t.data_ptr(), 8, t.data_ptr(), 16, t.data_ptr(), None,
                           None, 16, None, None, 0.0, None)
    assert rc == B.LGA_ERR_SHAPE
    rc = B.lib.lga_op_gemm(BF16, 0, 1, B.LGA_EPI_STORE, 8, 8, 8, t.data_ptr(), 8, t.data_ptr(), 8, t.data_ptr(), None,
                           None, 8, None, None, 0.0, None)
    assert rc == B.LGA_ERR_SHAPE                  # layout pair the layer never uses
    rc = B.lib.lga_op_gemm(F32, 1, 0, B.LGA_EPI_BIAS, 8, 8, 8, t.data_ptr(), 8, t.data_ptr(), 8, t.data_ptr(), None,
                           None, 8, None, None, 0.0, None)
    assert rc == B.LGA_ERR_ARG                    # bias missing
    torch.cuda.synchronize()


@pytest.mark.parametrize("dt,rows,d", [
    (F32, 37, 70), (F32, 5, 1), (BF16, 130, 256), (BF16, 33, 1000), (BF16, 3, 12288),
    # more rows than blocks (a block walks over several rows, requesting the next one early), every block size,
    # a ragged second pack, a row too wide for the row-walking kernels, the vector path of the fp32 mode
    (BF16, 5000, 3072), (BF16, 3000, 8192), (BF16, 700, 10000), (BF16, 40, 25600), (F32, 2500, 4096), (BF16, 2100, 768),
    (F16, 130, 256), (F16, 33, 1000), (F16, 5000, 3072), (F16, 40, 25600),
])
def test_layernorm_forward_and_backward(dt, rows, d):
    rng = np.random.default_rng(rows * 1000 + d)
    x = rnd(rng, (rows, d), dt, 2.0) + (0.5 if dt == F32 else 0.0)
    x = ROUND[dt](x)
    g = (1 + 0.3 * rng.standard_normal(d)).astype(np.float32)
    b = (0.2 * rng.standard_normal(d)).astype(np.float32)
    dy = rnd(rng, (rows, d), dt)
    resid = rnd(rng, (rows, d), dt)
    eps = 1e-5
    y_ref, xhat, rstd = O.layer_norm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), eps)
    dx_ref, dg_ref, db_ref = O.layer_norm_backward(dy.astype(np.float64), xhat, rstd, g.astype(np.float64))
    dx_ref = dx_ref + resid
    xd, dyd, rd = to_dev(x, dt), to_dev(dy, dt), to_dev(resid, dt)
    gd, bd = fvec(g), fvec(b)
    y, dx = empty_dev((rows, d), dt), empty_dev((rows, d), dt)
    mean, rs = torch.empty(rows, device="cuda"), torch.empty(rows, device="cuda")
    B.check(B.lib.lga_op_layernorm_fwd(dt, xd.data_ptr(), gd.data_ptr(), bd.data_ptr(), y.data_ptr(), mean.data_ptr(),
                                       rs.data_ptr(), rows, d, eps, None))
    old_g = rng.standard_normal(d).astype(np.float32); old_b = rng.standard_normal(d).astype(np.float32)
    dgd, dbd = fvec(old_g), fvec(old_b)
    scratch = torch.empty(int(B.lib.lga_op_layernorm_bwd_scratch_floats(rows, d)), device="cuda")
    B.check(B.lib.lga_op_layernorm_bwd(dt, dyd.data_ptr(), xd.data_ptr(), mean.data_ptr(), rs.data_ptr(), gd.data_ptr(),
                                       rd.data_ptr(), dx.data_ptr(), dgd.data_ptr(), dbd.data_ptr(), 1.0,
                                       scratch.data_ptr(), rows, d, None))
    torch.cuda.synchronize()
    tol = TOL_OUT[dt]
    assert rel_err(to_host(y), y_ref) < tol
    assert np.abs(mean.cpu().numpy() - x.astype(np.float64).mean(-1)).max() < 1e-5
    assert rel_err(rs.cpu().numpy(), rstd[:, 0]) < 1e-5
    assert rel_err(to_host(dx), dx_ref) < tol
    assert rel_err(dgd.cpu().numpy(), old_g + dg_ref) < 2e-5
    assert rel_err(dbd.cpu().numpy(), old_b + db_ref) < 2e-5


@pytest.mark.parametrize("dt,rows,cols,ld", [(F32, 300, 45, 50), (BF16, 1000, 264, 272), (BF16, 129, 8, 8), (F32, 0, 16, 16),
                                             (F16, 1000, 264, 272)])
def test_column_sums(dt, rows, cols, ld):
    rng = np.random.default_rng(rows + cols)
    a = rnd(rng, (max(rows, 1), ld), dt)[:rows]
    ad = to_dev(a if rows else np.zeros((1, ld), np.float32), dt)
    old = rng.standard_normal(cols).astype(np.float32)
    out = fvec(old)
    scratch = torch.empty(max(1, int(B.lib.lga_op_colsum_scratch_floats(rows, cols))), device="cuda")
    B.check(B.lib.lga_op_colsum(dt, ad.data_ptr(), rows, cols, ld, 1.0, out.data_ptr(), scratch.data_ptr(), None))
    torch.cuda.synchronize()
    ref = old.astype(np.float64) + a[:, :cols].astype(np.float64).sum(0)
    assert rel_err(out.cpu().numpy(), ref) < 1e-5
    B.check(B.lib.lga_op_colsum(dt, ad.data_ptr(), rows, cols, ld, 0.0, out.data_ptr(), scratch.data_ptr(), None))
    torch.cuda.synchronize()
    assert rel_err(out.cpu().numpy(), a[:, :cols].astype(np.float64).sum(0)) < 1e-5


def attention_reference(qkv, dout, n_seq, s, heads, dh, causal=True):
    d = heads * dh
    t = qkv.astype(np.float64).reshape(n_seq, s, 3, heads, dh)
    q, k, v = (t[:, :, i].transpose(0, 2, 1, 3) for i in range(3))
    out, prob = O.attention(q, k, v, causal)
    scores = (q @ np.swapaxes(k, -1, -2)) / math.sqrt(dh)
    if causal:
        mask = np.triu(np.ones((s, s), dtype=bool), 1)
        scores = np.where(mask, -np.inf, scores)
    mx = scores.max(-1, keepdims=True)
    lse = (mx + np.log(np.exp(scores - mx).sum(-1, keepdims=True)))[..., 0]
    do = dout.astype(np.float64).reshape(n_seq, s, heads, dh).transpose(0, 2, 1, 3)
    dq, dk, dv = O.causal_attention_backward(do, q, k, v, prob)
    merge = lambda z: z.transpose(0, 2, 1, 3).reshape(n_seq * s, d)
    return merge(out), lse, np.concatenate([merge(dq), merge(dk), merge(dv)], axis=1)


ATTN_CASES = [
    # dtype, kind, n_seq, s, heads, dh
    (F32, 0, 2, 37, 3, 16), (F32, 0, 1, 1, 1, 8), (BF16, 0, 2, 70, 2, 32),
    (BF16, 1, 2, 200, 2, 32), (BF16, 1, 1, 333, 3, 64), (BF16, 1, 2, 256, 2, 128), (BF16, 1, 1, 130, 2, 160),
    (BF16, 1, 1, 1, 1, 64), (BF16, 1, 3, 64, 1, 96),
    # long enough for the loops over fully visible tiles and for the LDS stages to wrap around, ragged ends
    (BF16, 1, 1, 1100, 2, 128), (BF16, 1, 2, 640, 1, 64), (BF16, 1, 1, 777, 1, 96), (BF16, 1, 1, 520, 1, 160),
    (BF16, 1, 1, 600, 1, 32),
    # head sizes between the kernels' own (32, 64, 96, 128, 160): run in the next larger kernel, extra columns as zeros
    (BF16, 1, 2, 200, 2, 152), (BF16, 1, 1, 333, 3, 72), (BF16, 1, 1, 130, 2, 8), (BF16, 1, 1, 97, 2, 40),
    (BF16, 1, 1, 300, 2, 104),
]
# the encoder variant (no mask): whole tiles, ragged last tiles of every residue class that matters (a last
# key block that is partly / wholly past the end), sequences shorter than a block, every head size
FULL_CASES = [
    (F32, 0, 2, 37, 3, 16), (F32, 0, 1, 1, 1, 8), (BF16, 0, 1, 70, 2, 32),
    (BF16, 1, 2, 256, 2, 128), (BF16, 1, 1, 333, 3, 64), (BF16, 1, 2, 200, 2, 32), (BF16, 1, 1, 130, 2, 160),
    (BF16, 1, 1, 1, 1, 64), (BF16, 1, 3, 64, 1, 96), (BF16, 1, 1, 31, 2, 128), (BF16, 1, 1, 97, 1, 64),
    (BF16, 1, 1, 1100, 2, 128), (BF16, 1, 2, 640, 1, 64), (BF16, 1, 1, 777, 1, 96), (BF16, 1, 1, 520, 1, 160),
    (BF16, 1, 1, 600, 1, 32), (BF16, 1, 2, 200, 2, 152), (BF16, 1, 1, 333, 3, 72), (BF16, 1, 1, 97, 2, 40),
]


@pytest.mark.parametrize("case", [c + (True,) for c in with_half(ATTN_CASES)] + [c + (False,) for c in with_half(FULL_CASES)],
                         ids=lambda c: "-".join(map(str, c[:-1])) + ("-causal" if c[-1] else "-full"))
def test_attention_forward_and_backward(case):
    dt, kind, n_seq, s, heads, dh, causal = case
    d = heads * dh
    rng = np.random.default_rng(hash(case[:-1]) % (2 ** 32))
    qkv = rnd(rng, (n_seq * s, 3 * d), dt)
    dout = rnd(rng, (n_seq * s, d), dt)
    out_ref, lse_ref, dqkv_ref = attention_reference(qkv, dout, n_seq, s, heads, dh, causal)
    qd, dod = to_dev(qkv, dt), to_dev(dout, dt)
    out, dqkv = empty_dev((n_seq * s, d), dt), empty_dev((n_seq * s, 3 * d), dt)
    lse = torch.empty(n_seq * heads * s, device="cuda")
    delta = torch.empty(n_seq * heads * s, device="cuda")
    B.check(B.lib.lga_op_attention_fwd(dt, kind, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, s, heads, dh,
                                       int(causal), None))
    B.check(B.lib.lga_op_attention_bwd(dt, kind, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), dod.data_ptr(),
                                       dqkv.data_ptr(), delta.data_ptr(), n_seq, s, heads, dh, int(causal), None))
    torch.cuda.synchronize()
    tol_f, tol_b = TOL_ATTN[dt]
    assert rel_err(to_host(out), out_ref) < tol_f
    assert np.abs(lse.cpu().numpy().reshape(n_seq, heads, s) - lse_ref).max() < (1e-5 if dt == F32 else 1e-3) * max(1.0, np.abs(lse_ref).max())
    got = to_host(dqkv)
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert rel_err(got[:, sl], dqkv_ref[:, sl]) < tol_b, name


@pytest.mark.parametrize("dt,dh,causal", [(BF16, 64, True), (BF16, 128, True), (BF16, 128, False), (F16, 64, True),
                                          (F16, 128, False), (F16, 160, True)])
def test_attention_with_scores_that_keep_growing_along_the_keys(dt, dh, causal):
    """The forward kernel fixes each query's softmax reference at its first 32 keys.  Here later keys score
    more than 100 (log2 units) above those, which the kernel must survive by starting over with a larger
    reference: outputs, log-sum-exp and the backward (which uses that log-sum-exp) still match the oracle.
    In half precision the probabilities must also stay below 65504, so the same happens after some 15 units."""
    n_seq, s, heads = 1, 320, 2
    d = heads * dh
    rng = np.random.default_rng(77 + dh)
    qkv = rng.standard_normal((n_seq * s, 3 * d)).astype(np.float32)
    ramp = 0.25 * np.arange(s, dtype=np.float32)                  # key j scores about j/4 nats with every query
    for h in range(heads):
        qkv[:, h * dh] = math.sqrt(dh)                            # q[:, 0] = sqrt(dh)
        qkv[:, d + h * dh] = ramp                                 # k[j, 0] = j / 4
    qkv = ROUND[dt](qkv)
    dout = rnd(rng, (n_seq * s, d), dt)
    out_ref, lse_ref, dqkv_ref = attention_reference(qkv, dout, n_seq, s, heads, dh, causal)
    # the case is what it claims: the last query's log-sum-exp lies > 100 log2 units above its first 32 scores
    t4 = qkv.astype(np.float64).reshape(n_seq, s, 3, heads, dh)
    first = np.einsum("bhc,bkhc->bhk", t4[:, -1, 0], t4[:, :32, 1]) / math.sqrt(dh)
    assert ((lse_ref[..., -1] - first.max(-1)) * math.log2(math.e) > 100).all()
    qd, dod = to_dev(qkv, dt), to_dev(dout, dt)
    out, dqkv = empty_dev((n_seq * s, d), dt), empty_dev((n_seq * s, 3 * d), dt)
    lse = torch.empty(n_seq * heads * s, device="cuda")
    delta = torch.empty(n_seq * heads * s, device="cuda")
    B.check(B.lib.lga_op_attention_fwd(dt, 1, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, s, heads, dh,
                                       int(causal), None))
    B.check(B.lib.lga_op_attention_bwd(dt, 1, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), dod.data_ptr(),
                                       dqkv.data_ptr(), delta.data_ptr(), n_seq, s, heads, dh, int(causal), None))
    torch.cuda.synchronize()
    assert np.isfinite(to_host(out)).all()
    assert rel_err(to_host(out), out_ref) < TOL_ATTN[dt][0]
    assert np.abs(lse.cpu().numpy().reshape(n_seq, heads, s) - lse_ref).max() < 1e-3 * np.abs(lse_ref).max()
    got = to_host(dqkv)
    # near one-hot probabilities times keys of size ~80: the rounding of dS weighs more than on ordinary inputs
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert rel_err(got[:, sl], dqkv_ref[:, sl]) < 2 * TOL_ATTN[dt][1], name


@pytest.mark.parametrize("dt,dh,s,causal", [(F16, 128, 2048, True), (F16, 64, 1000, False), (BF16, 128, 2048, True)])
def test_attention_with_the_score_spread_of_a_wide_layer(dt, dh, s, causal):
    """Queries and keys of size ~2.2 per element, as d_model = 12288 gives with N(0, 0.02^2) weights: scores spread
    by ~7 log2 units (one sigma), so among 2048 keys some lie 15 - 25 above the best of a query's first 32.  That
    is nothing for bf16 and beyond 65504 for half precision, whose kernel must then start over."""
    n_seq, heads = 1, 2
    d = heads * dh
    rng = np.random.default_rng(s + dh)
    qkv = rng.standard_normal((n_seq * s, 3 * d)).astype(np.float32)
    qkv[:, :2 * d] *= 2.2
    qkv = ROUND[dt](qkv)
    dout = rnd(rng, (n_seq * s, d), dt)
    out_ref, lse_ref, dqkv_ref = attention_reference(qkv, dout, n_seq, s, heads, dh, causal)
    t4 = qkv.astype(np.float64).reshape(n_seq, s, 3, heads, dh)
    sc = np.einsum("bqhc,bkhc->bhqk", t4[:, :, 0], t4[:, :, 1]) / math.sqrt(dh) * math.log2(math.e)
    if causal:
        sc = np.where(np.tril(np.ones((s, s), dtype=bool)), sc, -np.inf)
    assert ((sc.max(-1) - sc[..., :32].max(-1)) > 16).any()          # the case is what it claims
    qd, dod = to_dev(qkv, dt), to_dev(dout, dt)
    out, dqkv = empty_dev((n_seq * s, d), dt), empty_dev((n_seq * s, 3 * d), dt)
    lse = torch.empty(n_seq * heads * s, device="cuda")
    delta = torch.empty(n_seq * heads * s, device="cuda")
    B.check(B.lib.lga_op_attention_fwd(dt, 1, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, s, heads, dh,
                                       int(causal), None))
    B.check(B.lib.lga_op_attention_bwd(dt, 1, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), dod.data_ptr(),
                                       dqkv.data_ptr(), delta.data_ptr(), n_seq, s, heads, dh, int(causal), None))
    torch.cuda.synchronize()
    assert np.isfinite(to_host(out)).all()
    assert rel_err(to_host(out), out_ref) < TOL_ATTN[dt][0]
    assert np.abs(lse.cpu().numpy().reshape(n_seq, heads, s) - lse_ref).max() < 1e-3 * np.abs(lse_ref).max()
    got = to_host(dqkv)
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert rel_err(got[:, sl], dqkv_ref[:, sl]) < TOL_ATTN[dt][1], name


@pytest.mark.parametrize("dt,bad", [(BF16, float("nan")), (BF16, float("inf")), (F16, float("nan")), (F16, float("-inf"))])
def test_attention_forward_ends_on_non_finite_scores(dt, bad):
    """A query or key that is infinite or not a number makes its row sums non-finite, which no larger softmax
    reference can cure: the forward kernel gives up after a bounded number of attempts and returns a non-finite
    output for the (sequence, head) blocks concerned; the other head's output is untouched by it."""
    n_seq, s, heads, dh = 1, 300, 2, 64
    d = heads * dh
    rng = np.random.default_rng(5)
    qkv = rnd(rng, (n_seq * s, 3 * d), dt)
    dout = rnd(rng, (n_seq * s, d), dt)
    out_ref, _, _ = attention_reference(qkv, dout, n_seq, s, heads, dh, True)
    qkv[3, d + 5] = bad                                               # key 3 of head 0: seen by every query from 3 on
    qd = to_dev(qkv, dt)
    out = empty_dev((n_seq * s, d), dt)
    lse = torch.empty(n_seq * heads * s, device="cuda")
    B.check(B.lib.lga_op_attention_fwd(dt, 1, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, s, heads, dh, 1, None))
    torch.cuda.synchronize()
    got = to_host(out)
    if np.isnan(bad):
        assert not np.isfinite(got[3:, :dh]).any()                    # every query that sees the key
    else:
        assert not np.isfinite(got[3:, :dh]).all()                    # those whose score with it is +inf
    assert rel_err(got[:, dh:], out_ref[:, dh:]) < TOL_ATTN[dt][0]    # head 1
    assert rel_err(got[:3, :dh], out_ref[:3, :dh]) < TOL_ATTN[dt][0]  # queries before the bad key (causal)


@pytest.mark.parametrize("kind,dt,s,heads,dh,causal", [("fused", BF16, 16384, 1, 128, True), ("fused", BF16, 6000, 2, 64, False),
                                                       ("gemm", BF16, 4096, 2, 216, True), ("fused", F16, 8192, 1, 160, True)])
def test_attention_on_long_sequences(kind, dt, s, heads, dh, causal):
    """Sequences up to eight times the benchmark's 2048: dozens of query blocks per (sequence, head), hundreds of key
    tiles per block, the longest rows of the softmax sums."""
    n_seq, d = 1, heads * dh
    rng = np.random.default_rng(s + dh)
    qkv = rnd(rng, (n_seq * s, 3 * d), dt)
    dout = rnd(rng, (n_seq * s, d), dt)
    out_ref, lse_ref, dqkv_ref = attention_reference(qkv, dout, n_seq, s, heads, dh, causal)
    qd, dod = to_dev(qkv, dt), to_dev(dout, dt)
    out, dqkv = empty_dev((n_seq * s, d), dt), empty_dev((n_seq * s, 3 * d), dt)
    lse = torch.empty(n_seq * heads * s, device="cuda")
    delta = torch.empty(n_seq * heads * s, device="cuda")
    if kind == "fused":
        B.check(B.lib.lga_op_attention_fwd(dt, 1, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, s, heads, dh,
                                           int(causal), None))
        B.check(B.lib.lga_op_attention_bwd(dt, 1, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), dod.data_ptr(),
                                           dqkv.data_ptr(), delta.data_ptr(), n_seq, s, heads, dh, int(causal), None))
    else:
        nbytes = int(B.lib.lga_op_attention_gemm_workspace_bytes(s, heads))
        ws = torch.empty(nbytes // 4 + 64, device="cuda")
        base = (ws.data_ptr() + 255) // 256 * 256
        B.check(B.lib.lga_op_attention_gemm_fwd(dt, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, s, heads, dh,
                                                int(causal), base, nbytes, None))
        B.check(B.lib.lga_op_attention_gemm_bwd(dt, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), dod.data_ptr(),
                                                dqkv.data_ptr(), delta.data_ptr(), n_seq, s, heads, dh, int(causal), base,
                                                nbytes, None))
    torch.cuda.synchronize()
    tol_f, tol_b = TOL_ATTN[dt]
    assert rel_err(to_host(out), out_ref) < tol_f
    assert np.abs(lse.cpu().numpy().reshape(n_seq, heads, s) - lse_ref).max() < 1e-3 * max(1.0, np.abs(lse_ref).max())
    got = to_host(dqkv)
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert rel_err(got[:, sl], dqkv_ref[:, sl]) < tol_b, name


GEMM_ATTN_CASES = [
    # dtype, n_seq, s, heads, dh, causal, heads that fit the workspace
    (BF16, 2, 200, 3, 216, True, 3), (BF16, 1, 328, 2, 320, False, 2), (BF16, 1, 264, 3, 168, True, 1),
    (BF16, 1, 8, 1, 8, True, 1), (BF16, 1, 1024, 8, 176, True, 8), (BF16, 2, 136, 5, 64, False, 2),
    (F16, 2, 200, 3, 216, True, 2), (F16, 1, 520, 2, 320, False, 2),
]


@pytest.mark.parametrize("case", GEMM_ATTN_CASES, ids=lambda c: "-".join(map(str, c)))
def test_attention_built_from_batched_gemms(case):
    """Head sizes beyond the fused kernels (216 and 320 are the X_108 and X_160 heads of table B.1): scores through a
    workspace, batched GEMMs over the heads in all three operand layouts, row kernels for the softmax and for dS.
    Workspaces that hold all heads, some (several passes, a ragged last one) or one; 1024 x 8 heads takes the
    256 x 256-tile kernel for the score products, the others the 128 x 128 one."""
    dt, n_seq, s, heads, dh, causal, fit = case
    d = heads * dh
    rng = np.random.default_rng(hash(case) % (2 ** 32))
    qkv = rnd(rng, (n_seq * s, 3 * d), dt)
    dout = rnd(rng, (n_seq * s, d), dt)
    out_ref, lse_ref, dqkv_ref = attention_reference(qkv, dout, n_seq, s, heads, dh, causal)
    qd, dod = to_dev(qkv, dt), to_dev(dout, dt)
    out, dqkv = empty_dev((n_seq * s, d), dt), empty_dev((n_seq * s, 3 * d), dt)
    lse = torch.empty(n_seq * heads * s, device="cuda")
    delta = torch.empty(n_seq * heads * s, device="cuda")
    nbytes = int(B.lib.lga_op_attention_gemm_workspace_bytes(s, fit))
    assert nbytes == 12 * s * s * fit
    ws = torch.full((nbytes // 4 + 64,), float("nan"), device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    B.check(B.lib.lga_op_attention_gemm_fwd(dt, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, s, heads, dh,
                                            int(causal), base, nbytes, None))
    B.check(B.lib.lga_op_attention_gemm_bwd(dt, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), dod.data_ptr(),
                                            dqkv.data_ptr(), delta.data_ptr(), n_seq, s, heads, dh, int(causal), base,
                                            nbytes, None))
    torch.cuda.synchronize()
    tol_f, tol_b = TOL_ATTN[dt]
    assert rel_err(to_host(out), out_ref) < tol_f
    assert np.abs(lse.cpu().numpy().reshape(n_seq, heads, s) - lse_ref).max() < 1e-3 * max(1.0, np.abs(lse_ref).max())
    do64, o64 = dout.astype(np.float64).reshape(n_seq, s, heads, dh), out_ref.reshape(n_seq, s, heads, dh)
    assert rel_err(delta.cpu().numpy().reshape(n_seq, heads, s), (do64 * o64).sum(-1).transpose(0, 2, 1)) < tol_f
    got = to_host(dqkv)
    for name, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert rel_err(got[:, sl], dqkv_ref[:, sl]) < tol_b, name
    # refused on the host: sequence length or head size not a multiple of 8, workspace missing, unaligned or too small
    for bad in (dict(s=s + 4), dict(dh=dh + 4), dict(ws=None), dict(ws=base + 16), dict(nbytes=12 * s * s - 1)):
        a = dict(s=s, dh=dh, ws=base, nbytes=nbytes)
        a.update(bad)
        rc = B.lib.lga_op_attention_gemm_fwd(dt, qd.data_ptr(), out.data_ptr(), lse.data_ptr(), n_seq, a["s"], heads, a["dh"],
                                             int(causal), a["ws"], a["nbytes"], None)
        assert rc in (B.LGA_ERR_SHAPE, B.LGA_ERR_ARG), bad


def test_attention_mfma_rejects_unsupported_head_size():
    t = torch.zeros(4096, device="cuda", dtype=torch.bfloat16)
    l = torch.zeros(64, device="cuda")
    for dh in (168, 320, 12):            # above 160, or not a multiple of 8
        rc = B.lib.lga_op_attention_fwd(BF16, 1, t.data_ptr(), t.data_ptr(), l.data_ptr(), 1, 4, 1, dh, 1, None)
        assert rc == B.LGA_ERR_SHAPE
    rc = B.lib.lga_op_attention_fwd(F32, 1, t.data_ptr(), t.data_ptr(), l.data_ptr(), 1, 4, 1, 64, 1, None)
    assert rc == B.LGA_ERR_SHAPE


@pytest.mark.parametrize("n,with16", [(1003, BF16), (4096, BF16), (7, None), (0, None), (1003, F16), (4100, F16)])
def test_adam_kernel_against_closed_form(n, with16):
    rng = np.random.default_rng(n)
    w = rng.standard_normal(n).astype(np.float32)
    m = (0.1 * rng.standard_normal(n)).astype(np.float32)
    v = (0.01 * rng.random(n)).astype(np.float32)
    g = rng.standard_normal(n).astype(np.float32)
    hp = B.lga_adam(3e-3, 0.9, 0.999, 1e-8, 7)
    ohp = O.AdamHyper(lr=float(np.float32(3e-3)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)),
                      eps=float(np.float32(1e-8)), step=7)
    w_ref, m_ref, v_ref = O.adam_update(w.astype(np.float64), m.astype(np.float64), v.astype(np.float64),
                                        g.astype(np.float64), ohp)
    wd, md, vd, gd = fvec(w), fvec(m), fvec(v), fvec(g)
    w16 = empty_dev((max(n, 1),), with16 or BF16).zero_()
    import ctypes
    B.check(B.lib.lga_op_adam(wd.data_ptr(), md.data_ptr(), vd.data_ptr(), gd.data_ptr(),
                              w16.data_ptr() if with16 else None, with16 or 0, n, ctypes.byref(hp), None, None))
    torch.cuda.synchronize()
    if n == 0:
        return
    assert rel_err(wd.cpu().numpy(), w_ref) < 1e-6
    assert rel_err(md.cpu().numpy(), m_ref) < 1e-6
    assert rel_err(vd.cpu().numpy(), v_ref) < 1e-6
    if with16:
        assert np.array_equal(to_host(w16)[:n], ROUND[with16](wd.cpu().numpy()).astype(np.float64))


def test_adam_kernel_hand_worked_values():
    # same numbers as the oracle's pin: w=0.5 m=0.1 v=0.04 g=-0.2 lr=0.01 b1=0.9 b2=0.99 t=2 -> w'=0.49740139...
    import ctypes
    wd, md, vd, gd = fvec([0.5]), fvec([0.1]), fvec([0.04]), fvec([-0.2])
    hp = B.lga_adam(0.01, 0.9, 0.99, 1e-8, 2)
    B.check(B.lib.lga_op_adam(wd.data_ptr(), md.data_ptr(), vd.data_ptr(), gd.data_ptr(), None, 0, 1, ctypes.byref(hp), None,
                              None))
    torch.cuda.synchronize()
    assert abs(float(wd[0]) - 0.4974013907589168) < 2e-7
    assert abs(float(md[0]) - 0.07) < 1e-7 and abs(float(vd[0]) - 0.04) < 1e-7


@pytest.mark.parametrize("n,bad_at,bad", [(5000, 4999, float("inf")), (5000, 0, float("nan")), (4099, 4098, float("-inf")),
                                          (3, 1, float("nan")), (5000, None, 0.0)])
def test_adam_kernel_with_loss_scale_and_non_finite_test(n, bad_at, bad):
    """Gradient scaling (section 2.2): the gradient is divided by the loss scale; with skip_nonfinite one infinity or
    NaN anywhere in it (first element, last element of the vector part, scalar tail) leaves the whole update out."""
    import ctypes
    rng = np.random.default_rng(n)
    w = rng.standard_normal(n).astype(np.float32)
    m = (0.1 * rng.standard_normal(n)).astype(np.float32)
    v = (0.01 * rng.random(n)).astype(np.float32)
    scale = 512.0
    g = (scale * rng.standard_normal(n)).astype(np.float32)
    if bad_at is not None:
        g[bad_at] = bad
    hp = B.lga_adam(3e-3, 0.9, 0.999, 1e-8, 7, scale, 1)
    ohp = O.AdamHyper(lr=float(np.float32(3e-3)), beta1=float(np.float32(0.9)), beta2=float(np.float32(0.999)),
                      eps=float(np.float32(1e-8)), step=7, loss_scale=scale, skip_nonfinite=True)
    w_ref, m_ref, v_ref = O.adam_update(w.astype(np.float64), m.astype(np.float64), v.astype(np.float64),
                                        g.astype(np.float64), ohp)
    wd, md, vd, gd = fvec(w), fvec(m), fvec(v), fvec(g)
    w16 = empty_dev((n,), F16).fill_(3.0)
    flag = torch.full((1,), 77, device="cuda", dtype=torch.int32)
    assert B.lib.lga_op_adam(wd.data_ptr(), md.data_ptr(), vd.data_ptr(), gd.data_ptr(), w16.data_ptr(), F16, n,
                             ctypes.byref(hp), None, None) == B.LGA_ERR_ARG         # the flag is required
    B.check(B.lib.lga_op_adam(wd.data_ptr(), md.data_ptr(), vd.data_ptr(), gd.data_ptr(), w16.data_ptr(), F16, n,
                              ctypes.byref(hp), flag.data_ptr(), None))
    torch.cuda.synchronize()
    assert int(flag[0]) == (1 if bad_at is not None else 0)
    if bad_at is not None:
        assert O.adam_skips(g, ohp)
        assert np.array_equal(wd.cpu().numpy(), w) and np.array_equal(md.cpu().numpy(), m) and np.array_equal(vd.cpu().numpy(), v)
        assert np.all(to_host(w16) == 3.0)
    else:
        assert rel_err(wd.cpu().numpy(), w_ref) < 1e-6
        assert rel_err(md.cpu().numpy(), m_ref) < 1e-6
        assert rel_err(vd.cpu().numpy(), v_ref) < 1e-6
        assert np.array_equal(to_host(w16), S.round_to_fp16(wd.cpu().numpy()).astype(np.float64))
