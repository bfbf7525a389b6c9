"""Attention kernels on a sequence so long (131200 tokens, 1025 blocks of 128) that the (block, chunk) pairs no
longer fit the kernels' work table, so that they run on their blocks x chunks grid.  The oracle cannot form the
whole score matrix at this length; it follows sampled query rows one by one (a causal row i is an ordinary
attention of one query over keys 0 .. i), and the upstream gradient is non-zero only on sampled rows, which
makes dK and dV sums of those rows' contributions: every key block and every chunk of the grid is compared."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import synth
from oracle import stp_oracle as O
from harness import to_dev, to_host, rel_err


def test_attention_on_the_grid_fallback_matches_sampled_oracle_rows():
    seq, n, d = 131200, 1, 64
    wl = synth.Workload("long", 64, n, d, 64, seq, 1)
    desc = stp.make_desc(wl)
    for kind in (stp.ATTN_FWD, stp.ATTN_DKV, stp.ATTN_DQ):
        assert stp.attention_plan(desc, kind)[2] == [], "this shape is meant to exceed the work table"
    rng = np.random.default_rng(131200)
    qkv = synth.quantize(rng.standard_normal((seq, 3 * d), dtype=np.float32), "bf16")
    rows_fwd = sorted({0, 1, 127, 128, 129, 8191, 8192, 67199, 67200, seq - 129, seq - 128, seq - 1} |
                      {int(x) for x in rng.integers(0, seq, 36)})
    rows_bwd = sorted(set(rows_fwd[::4]) | {seq - 1})
    dctx = np.zeros((seq, d), dtype=np.float32)
    dctx[rows_bwd] = synth.quantize(rng.standard_normal((len(rows_bwd), d), dtype=np.float32), "bf16")

    ctx = stp.Context(0)
    import ctypes as C
    nbytes = C.c_size_t()
    assert stp.lib().stp_workspace_bytes(C.byref(desc), C.byref(nbytes)) == 0
    ctx.set_workspace(torch.empty(nbytes.value, dtype=torch.uint8, device="cuda"))
    qkvd, dctxd = to_dev(qkv, "bf16"), to_dev(dctx, "bf16")
    out = torch.zeros((seq, d), dtype=qkvd.dtype, device="cuda")
    lse = torch.zeros((1, n, seq), dtype=torch.float32, device="cuda")
    delta = torch.zeros_like(lse)
    dqkv = torch.zeros_like(qkvd)
    print("launching forward and backward at seq", seq, flush=True)
    ctx.attention_forward(desc, qkvd, out, lse)
    ctx.attention_backward(desc, qkvd, out, lse, dctxd, delta, dqkv)
    torch.cuda.synchronize()
    print("GPU done; oracle rows", flush=True)
    got_o, got_l, got_d = to_host(out), to_host(lse)[0, 0], to_host(dqkv)
    ctx.close()

    q64 = qkv.astype(np.float64)
    Q, K, V = q64[:, :d], q64[:, d:2 * d], q64[:, 2 * d:]
    tol = 1e-2
    for i in rows_fwd:
        ref = O.attention_fwd(Q[i:i + 1, None, :], K[:i + 1, None, :], V[:i + 1, None, :], False)[0, 0]
        assert np.max(np.abs(got_o[i] - ref)) <= tol * max(1.0, np.max(np.abs(ref))), i
        s = K[:i + 1] @ Q[i] / np.sqrt(d)
        assert abs(got_l[i] - (s.max() + np.log(np.exp(s - s.max()).sum()))) < 2e-2, i
    dk_ref, dv_ref = np.zeros((seq, d)), np.zeros((seq, d))
    dq_ref = np.zeros((seq, d))
    for i in rows_bwd:
        dq, dk, dv = O.attention_bwd(Q[i:i + 1, None, :], K[:i + 1, None, :], V[:i + 1, None, :],
                                     dctx[i:i + 1, None, :].astype(np.float64), False)
        dq_ref[i] = dq[0, 0]
        dk_ref[:i + 1] += dk[:, 0]
        dv_ref[:i + 1] += dv[:, 0]
    assert rel_err(got_d[:, :d], dq_ref) < tol            # rows without an upstream gradient are zero in both
    assert not got_d[[r for r in range(0, seq, 997) if r not in rows_bwd], :d].any()
    assert rel_err(got_d[:, d:2 * d], dk_ref) < tol
    assert rel_err(got_d[:, 2 * d:], dv_ref) < tol
