"""lga_op_colsum_static - the column sums for callers that cannot allocate - against lga_op_colsum through the C ABI.

Two calls in a row on the same GPU, the second on a smaller input, so that the built-in scratch still holds the first
call's partial sums when the second runs: both must equal lga_op_colsum's output bit for bit (same two kernels) and
the fp64 column sums to the fp32 gate.  Sizes beyond the built-in scratch are refused on the host.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import synth_inputs as S
from paper_2106_02679_amd import binding as B
from gpu_helpers import to_dev, rel_err

F32, BF16, F16 = B.LGA_FP32, B.LGA_BF16, B.LGA_FP16
ROUND = {F32: lambda a: a, BF16: S.round_to_bf16, F16: S.round_to_fp16}


def _both(dt, a, cols, ld, beta, old):
    """(workspace entry point's result, static entry point's result) on the same input."""
    rows = a.shape[0]
    ad = to_dev(a, dt)
    res = []
    ws = torch.empty(max(1, int(B.lib.lga_op_colsum_scratch_floats(rows, cols))), device="cuda")
    out = torch.from_numpy(old.copy()).cuda()
    B.check(B.lib.lga_op_colsum(dt, ad.data_ptr(), rows, cols, ld, beta, out.data_ptr(), ws.data_ptr(), None))
    torch.cuda.synchronize()
    res.append(out.cpu().numpy())
    out = torch.from_numpy(old.copy()).cuda()
    B.check(B.lib.lga_op_colsum_static(dt, ad.data_ptr(), rows, cols, ld, beta, out.data_ptr(), None))
    torch.cuda.synchronize()
    res.append(out.cpu().numpy())
    return res


@pytest.mark.parametrize("dt", [F32, BF16, F16])
def test_static_scratch_column_sums_match_the_workspace_entry_point_on_two_calls_in_a_row(dt):
    rng = np.random.default_rng(7 + dt)
    # first call: 1300 rows (11 row chunks, the last ragged) x 1048 columns of a 1056-wide matrix; second: smaller in
    # both directions, so most of the scratch keeps the first call's partial sums while it runs
    for rows, cols, ld, beta in ((1300, 1048, 1056, 1.0), (300, 264, 272, 0.0), (129, 8, 8, 1.0)):
        a = ROUND[dt]((rng.standard_normal((rows, ld))).astype(np.float32))
        old = rng.standard_normal(cols).astype(np.float32)
        ws, st = _both(dt, a, cols, ld, beta, old)
        assert np.array_equal(ws, st), (rows, cols)
        ref = beta * old.astype(np.float64) + a[:, :cols].astype(np.float64).sum(0)
        assert rel_err(st, ref) < 1e-5, (rows, cols)


def test_static_scratch_limit_is_enforced_on_the_host():
    limit = int(B.lib.lga_op_colsum_static_max_floats())
    assert limit == 4 << 20
    rows, cols = 8192, 36864                       # 64 chunks x 2 x 36864 floats: beyond the built-in scratch
    assert int(B.lib.lga_op_colsum_scratch_floats(rows, cols)) > limit
    a = torch.zeros(8, device="cuda")              # never read: the call is refused before any launch
    out = torch.zeros(cols, device="cuda")
    rc = B.lib.lga_op_colsum_static(F32, a.data_ptr(), rows, cols, cols, 0.0, out.data_ptr(), None)
    assert rc == B.LGA_ERR_SHAPE and "built-in scratch" in B.last_error()
    # the largest size that fits runs: 128 rows per chunk
    cols = 4096
    rows = 128 * (limit // (2 * cols))
    assert int(B.lib.lga_op_colsum_scratch_floats(rows, cols)) == limit
    big = torch.ones((rows, cols), device="cuda")
    out = torch.zeros(cols, device="cuda")
    B.check(B.lib.lga_op_colsum_static(F32, big.data_ptr(), rows, cols, cols, 0.0, out.data_ptr(), None))
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), np.full(cols, float(rows), np.float32))
