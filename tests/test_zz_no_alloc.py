"""The entry point that allocates nothing: stp_colsum_noalloc keeps its partial sums in a fixed array of the
library's device image.  It must give the same bits as stp_colsum (same kernels) on two calls in a row, the
second with a smaller input (what the first call left in the array must not be seen), and match the oracle."""
import numpy as np
import pytest
import torch

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import synth
from tests.harness import rel_err, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_colsum_noalloc_matches_colsum_on_two_calls_in_a_row(dtype):
    ctx = stp.Context(0)
    code = stp.BF16 if dtype == "bf16" else stp.F32
    rng = np.random.default_rng(7)
    # the second call is smaller in both extents, ragged in rows (not a multiple of 64) and in columns (not of 256)
    for T, N, scale in [(6144, 4096, 0.125), (1000, 264, 1.0)]:
        x_host = rng.standard_normal((T, N)).astype(np.float32)
        x_host = synth.quantize(x_host, dtype)
        x = to_dev(x_host, dtype)
        start = rng.standard_normal(N).astype(np.float32)
        out_ws = torch.from_numpy(start.copy()).cuda()
        out_na = torch.from_numpy(start.copy()).cuda()
        # reference entry point: partials in a workspace lane
        ws = torch.empty(3 * (((T + 63) // 64) * N * 4 + 256) + 256, dtype=torch.uint8, device="cuda")
        ctx.set_workspace(ws)
        ctx.colsum(code, T, N, x, scale, out_ws)
        ctx.set_workspace(None)          # the no-allocation entry point must not need one
        ctx.colsum_noalloc(code, T, N, x, scale, out_na)
        torch.cuda.synchronize()
        assert torch.equal(out_ws, out_na), (dtype, T, N)
        # the plain definition of the bias gradient: scale * sum over the token rows (the values are exact in
        # either storage type, the sums are fp32 on the device)
        ref = start.astype(np.float64) + scale * x_host.astype(np.float64).sum(0)
        assert rel_err(to_host(out_na), ref) < 1e-5
    ctx.close()


def test_colsum_noalloc_rejects_sizes_beyond_its_scratch():
    ctx = stp.Context(0)
    T, N = 64 * 1024, 2048            # 1024 patches of 64 rows x 2048 columns = 2 Mi partial sums > 1 Mi
    x = torch.zeros(8, dtype=torch.bfloat16, device="cuda")   # never read: the size check comes first
    out = torch.zeros(N, dtype=torch.float32, device="cuda")
    with pytest.raises(stp.StpError) as e:
        ctx.colsum_noalloc(stp.BF16, T, N, x, 1.0, out)
    assert e.value.status == 4
    ctx.close()
