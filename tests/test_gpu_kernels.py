"""Per-kernel parity against pieces of the fp64 oracle, through the C ABI."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import synth
from oracle import stp_oracle as O
from harness import to_dev, to_host, rel_err, TOL


@pytest.fixture(scope="module")
def ctx():
    c = stp.Context(0)
    c.set_workspace(torch.empty(256 << 20, dtype=torch.uint8, device="cuda"))
    yield c
    torch.cuda.synchronize()
    c.close()


def q(x, dtype):
    return synth.quantize(x, dtype)


# ------------------------------------------------------------------ GEMM
GEMM_SHAPES = [(128, 128, 64), (256, 256, 128), (384, 520, 200), (1000, 264, 72), (520, 1288, 328), (8, 8, 8)]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("a_trans,b_trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_layouts(ctx, dtype, a_trans, b_trans, M, N, K):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    A = q(rng.standard_normal((M, K), dtype=np.float32), dtype)
    B = q(rng.standard_normal((K, N), dtype=np.float32) * 0.05, dtype)
    Ad = to_dev(np.ascontiguousarray(A.T) if a_trans else A, dtype)
    Bd = to_dev(np.ascontiguousarray(B.T) if b_trans else B, dtype)
    Cd = torch.zeros((M, N), dtype=Ad.dtype, device="cuda")
    g = stp.GemmArgs(dtype=stp.BF16 if dtype == "bf16" else stp.F32, M=M, N=N, K=K,
                     A=Ad.data_ptr(), lda=M if a_trans else K, a_trans=a_trans,
                     B=Bd.data_ptr(), ldb=K if b_trans else N, b_trans=b_trans,
                     C=Cd.data_ptr(), ldc=N, bias_scale=1.0, resid_scale=1.0)
    ctx.gemm(g)
    torch.cuda.synchronize()
    ref = A.astype(np.float64) @ B.astype(np.float64)
    assert rel_err(to_host(Cd), ref) < (4e-3 if dtype == "bf16" else 2e-6)


@pytest.mark.parametrize("tile", [(256, 256), (256, 128), (128, 256), (128, 128)])
@pytest.mark.parametrize("a_trans,b_trans", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("M,N,K", [(520, 776, 160), (264, 136, 32), (1288, 520, 352)])
def test_gemm_forced_tiles(ctx, tile, a_trans, b_trans, M, N, K):
    """Every workgroup tile of the direct-to-LDS kernel, on shapes with ragged edge tiles, fewer K-tiles than
    pipeline stages (K = 32) and more (K = 352)."""
    rng = np.random.default_rng(M + N + K)
    A = q(rng.standard_normal((M, K), dtype=np.float32), "bf16")
    B = q(rng.standard_normal((K, N), dtype=np.float32) * 0.05, "bf16")
    Ad = to_dev(np.ascontiguousarray(A.T) if a_trans else A, "bf16")
    Bd = to_dev(np.ascontiguousarray(B.T) if b_trans else B, "bf16")
    Cd = torch.zeros((M, N), dtype=Ad.dtype, device="cuda")
    ctx.gemm(stp.GemmArgs(dtype=stp.BF16, M=M, N=N, K=K, A=Ad.data_ptr(), lda=M if a_trans else K, a_trans=a_trans,
                          B=Bd.data_ptr(), ldb=K if b_trans else N, b_trans=b_trans, C=Cd.data_ptr(), ldc=N,
                          bias_scale=1.0, resid_scale=1.0, tile_m=tile[0], tile_n=tile[1]))
    torch.cuda.synchronize()
    assert rel_err(to_host(Cd), A.astype(np.float64) @ B.astype(np.float64)) < 4e-3


@pytest.mark.parametrize("b_trans", [0, 1])
@pytest.mark.parametrize("M,N,K", [(520, 776, 160), (264, 136, 32), (1288, 520, 352), (192, 256, 64), (1928, 264, 96)])
def test_gemm_192_row_tile(ctx, b_trans, M, N, K):
    """The 192 x 256 tile (k-contiguous A only): 12 one-KB pieces of A per K-tile for 8 waves, so half of the
    waves have an unused load slot; ragged last tile rows (M = 520: 136 of 192; M = 1928: 8 of 192).  Same
    bits as the 256 x 256 tile: the accumulation order over K does not depend on the tile."""
    rng = np.random.default_rng(M + N + K + 1)
    A = q(rng.standard_normal((M, K), dtype=np.float32), "bf16")
    B = q(rng.standard_normal((K, N), dtype=np.float32) * 0.05, "bf16")
    Ad = to_dev(A, "bf16")
    Bd = to_dev(np.ascontiguousarray(B.T) if b_trans else B, "bf16")
    out = {}
    for tile in ((192, 256), (256, 256)):
        Cd = torch.zeros((M, N), dtype=Ad.dtype, device="cuda")
        ctx.gemm(stp.GemmArgs(dtype=stp.BF16, M=M, N=N, K=K, A=Ad.data_ptr(), lda=K, B=Bd.data_ptr(),
                              ldb=K if b_trans else N, b_trans=b_trans, C=Cd.data_ptr(), ldc=N, bias_scale=1.0,
                              resid_scale=1.0, tile_m=tile[0], tile_n=tile[1]))
        torch.cuda.synchronize()
        out[tile] = Cd
    assert rel_err(to_host(out[(192, 256)]), A.astype(np.float64) @ B.astype(np.float64)) < 4e-3
    assert torch.equal(out[(192, 256)], out[(256, 256)])


@pytest.mark.parametrize("dtype,tile", [("bf16", (0, 0)), ("f32", (0, 0)), ("bf16", (256, 256)), ("bf16", (128, 128)),
                                        ("bf16", (256, 128)), ("bf16", (128, 256)), ("bf16", (192, 256))])
def test_gemm_epilogues(ctx, dtype, tile):
    M, N, K = (392, 456, 136) if tile == (0, 0) else (392, 456, 160)
    rng = np.random.default_rng(5)
    tol = 6e-3 if dtype == "bf16" else 3e-6
    A = q(rng.standard_normal((M, K), dtype=np.float32), dtype)
    B = q(rng.standard_normal((K, N), dtype=np.float32) * 0.1, dtype)
    bias = q(rng.standard_normal(N, dtype=np.float32), dtype)
    R = q(rng.standard_normal((M, N), dtype=np.float32), dtype)
    Ad, Bd, bd, Rd = (to_dev(x, dtype) for x in (A, B, bias, R))
    code = stp.BF16 if dtype == "bf16" else stp.F32
    base = dict(dtype=code, M=M, N=N, K=K, A=Ad.data_ptr(), lda=K, B=Bd.data_ptr(), ldb=N, ldc=N, tile_m=tile[0],
                tile_n=tile[1])
    AB = A.astype(np.float64) @ B.astype(np.float64)
    # bias*scale + resid*scale
    Cd = torch.zeros((M, N), dtype=Ad.dtype, device="cuda")
    ctx.gemm(stp.GemmArgs(**base, C=Cd.data_ptr(), bias=bd.data_ptr(), bias_scale=0.25, resid=Rd.data_ptr(), ldr=N,
                          resid_scale=0.125))
    torch.cuda.synchronize()
    assert rel_err(to_host(Cd), AB + 0.25 * bias + 0.125 * R) < tol
    # dual output: C = v, C2 = gelu(v)
    C2 = torch.zeros_like(Cd)
    ctx.gemm(stp.GemmArgs(**base, C=Cd.data_ptr(), bias=bd.data_ptr(), bias_scale=1.0, resid_scale=1.0, epilogue=1,
                          C2=C2.data_ptr(), ld2=N))
    torch.cuda.synchronize()
    assert rel_err(to_host(Cd), AB + bias) < tol
    assert rel_err(to_host(C2), O.gelu(AB + bias)) < tol
    # C = v * gelu'(aux)
    ctx.gemm(stp.GemmArgs(**base, C=Cd.data_ptr(), bias_scale=1.0, resid_scale=1.0, epilogue=2, aux=Rd.data_ptr(), ld2=N))
    torch.cuda.synchronize()
    assert rel_err(to_host(Cd), AB * O.gelu_grad(R.astype(np.float64))) < tol
    # fp32 accumulate: C32 += v, twice
    C32 = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    for _ in range(2):
        ctx.gemm(stp.GemmArgs(**base | dict(ldc=N), C=C32.data_ptr(), c_f32_accum=1, bias_scale=1.0, resid_scale=1.0))
    torch.cuda.synchronize()
    assert rel_err(to_host(C32), 0.5 + 2 * AB) < (3e-6 if dtype == "f32" else 1e-5)


def test_gemm_operand_of_two_gib_takes_the_fallback_kernel(ctx):
    """An A operand of 2 GiB or more cannot be addressed with the 32-bit offsets of the direct-to-LDS kernel; the
    library must fall back to the register-staged kernel (K a multiple of 32, so only the size decides).
    Checked on sampled rows, including the last ones (past the 2 GiB mark)."""
    M, N, K = 264200, 64, 4096                      # A: 264200 x 4096 bf16 = 2.16 GB
    g = torch.Generator(device="cuda").manual_seed(3)
    A = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    Bm = (torch.randn((K, N), generator=g, device="cuda", dtype=torch.float32) * 0.05).to(torch.bfloat16)
    Cd = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    ctx.gemm(stp.GemmArgs(dtype=stp.BF16, M=M, N=N, K=K, A=A.data_ptr(), lda=K, B=Bm.data_ptr(), ldb=N, C=Cd.data_ptr(),
                          ldc=N, bias_scale=1.0, resid_scale=1.0))
    torch.cuda.synchronize()
    rows = [0, 1, 255, 256, 131071, 262143, 262144, 262145, M - 2, M - 1]
    ref = to_host(A[rows]) @ to_host(Bm)
    assert rel_err(to_host(Cd[rows]), ref) < 4e-3


def test_gemm_rejects_bad_arguments(ctx):
    x = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    ok = dict(dtype=stp.BF16, M=64, N=64, K=64, A=x.data_ptr(), lda=64, B=x.data_ptr(), ldb=64, C=x.data_ptr(), ldc=64)
    for bad, status in [(dict(M=63), 2), (dict(A=None), 1), (dict(A=x.data_ptr() + 2), 3), (dict(lda=32), 2),
                        (dict(dtype=7), 1), (dict(epilogue=1), 1), (dict(tile_m=64, tile_n=128), 1),
                        (dict(tile_m=128, tile_n=0), 1), (dict(K=40, lda=64, tile_m=128, tile_n=128), 1),
                        (dict(tile_m=192, tile_n=128), 1), (dict(tile_m=192, tile_n=256, a_trans=1), 1),
                        (dict(dtype=stp.F32, tile_m=128, tile_n=128), 1)]:
        with pytest.raises(stp.StpError) as e:
            ctx.gemm(stp.GemmArgs(**(ok | bad)))
        assert e.value.status == status
    ctx.gemm(stp.GemmArgs(**(ok | dict(M=0))))  # empty problem is a no-op


# ------------------------------------------------------------------ norms
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("norm", ["ln", "rms"])
@pytest.mark.parametrize("T,h", [(37, 256), (130, 4096), (64, 5120), (9, 1024), (5, 8), (600, 2056), (24, 8192)])
def test_norm_forward_backward(ctx, dtype, norm, T, h):
    rng = np.random.default_rng(T + h)
    cfg = O.LayerCfg(h, 1, 8, 8, norm=norm)
    x = q(rng.standard_normal((T, h), dtype=np.float32) * 2 + 0.5, dtype)
    gam = q(1 + 0.1 * rng.standard_normal(h, dtype=np.float32), dtype)
    bet = q(0.1 * rng.standard_normal(h, dtype=np.float32), dtype)
    dy = q(rng.standard_normal((T, h), dtype=np.float32), dtype)
    dres = q(rng.standard_normal((T, h), dtype=np.float32), dtype)
    xd, gd, bd, dyd, drd = (to_dev(v, dtype) for v in (x, gam, bet, dy, dres))
    y = torch.empty_like(xd)
    stats = torch.empty((T, 2), dtype=torch.float32, device="cuda")
    code = stp.BF16 if dtype == "bf16" else stp.F32
    ncode = stp.NORM_LN if norm == "ln" else stp.NORM_RMS
    ctx.norm_forward(code, ncode, T, h, cfg.eps, xd, gd, bd if norm == "ln" else None, y, stats)
    torch.cuda.synchronize()
    ref = O.norm_fwd(cfg, x.astype(np.float64), gam.astype(np.float64), bet.astype(np.float64) if norm == "ln" else None)
    tol = 8e-3 if dtype == "bf16" else 2e-6
    assert rel_err(to_host(y), ref) < tol
    dx = torch.empty_like(xd)
    dgam = torch.full((h,), 1.0, dtype=torch.float32, device="cuda")
    dbet = torch.full((h,), -1.0, dtype=torch.float32, device="cuda")
    ctx.norm_backward(code, ncode, T, h, xd, gd, stats, dyd, drd, dx, dgam, dbet, lane=1)
    torch.cuda.synchronize()
    rdx, rdg, rdb = O.norm_bwd(cfg, dy.astype(np.float64), x.astype(np.float64), gam.astype(np.float64))
    assert rel_err(to_host(dx), rdx + dres) < tol
    assert rel_err(to_host(dgam), 1.0 + rdg) < 1e-5
    if norm == "ln":
        assert rel_err(to_host(dbet), -1.0 + rdb) < 1e-5
    # the same pass also hands out the scaled column sum of the residual-path gradient (the row-parallel bias
    # gradient of the unit above: (1/t) * sum over tokens, Eq. 1); dx and the norm gradients keep their bits
    dx2, rsum = torch.empty_like(xd), torch.full((h,), 0.5, dtype=torch.float32, device="cuda")
    dgam2 = torch.full((h,), 1.0, dtype=torch.float32, device="cuda")
    dbet2 = torch.full((h,), -1.0, dtype=torch.float32, device="cuda")
    ctx.norm_backward(code, ncode, T, h, xd, gd, stats, dyd, drd, dx2, dgam2, dbet2, lane=2, d_resid_sum=rsum,
                      d_resid_sum_scale=0.25)
    torch.cuda.synchronize()
    assert torch.equal(dx2, dx) and torch.equal(dgam2, dgam)
    assert rel_err(to_host(rsum), 0.5 + 0.25 * dres.astype(np.float64).sum(0)) < 1e-5
    rsum.fill_(0.0)
    ctx.norm_backward(code, ncode, T, h, xd, gd, stats, dyd, drd, dx2, None, None, d_resid_sum=rsum)
    torch.cuda.synchronize()
    assert torch.equal(dx2, dx)
    assert rel_err(to_host(rsum), dres.astype(np.float64).sum(0)) < 1e-5
    # no residual, no parameter gradients
    ctx.norm_backward(code, ncode, T, h, xd, gd, stats, dyd, None, dx, None, None)
    torch.cuda.synchronize()
    assert rel_err(to_host(dx), rdx) < tol


# ------------------------------------------------------------------ activations, rope, colsum
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_activations(ctx, dtype):
    n = 8 * 12345
    rng = np.random.default_rng(1)
    code = stp.BF16 if dtype == "bf16" else stp.F32
    tol = 8e-3 if dtype == "bf16" else 2e-6
    x, u, dy = (q(rng.standard_normal(n, dtype=np.float32) * 2, dtype) for _ in range(3))
    xd, ud, dyd = (to_dev(v, dtype) for v in (x, u, dy))
    y, y2 = torch.empty_like(xd), torch.empty_like(xd)
    ctx.gelu_forward(code, n, xd, y)
    ctx.gelu_backward(code, n, xd, dyd, y2)
    torch.cuda.synchronize()
    x64, u64, dy64 = (v.astype(np.float64) for v in (x, u, dy))
    assert rel_err(to_host(y), O.gelu(x64)) < tol
    assert rel_err(to_host(y2), dy64 * O.gelu_grad(x64)) < tol
    ctx.swiglu_forward(code, n, xd, ud, y)
    torch.cuda.synchronize()
    assert rel_err(to_host(y), O.silu(x64) * u64) < tol
    ctx.swiglu_backward(code, n, xd, ud, dyd, y, y2)
    torch.cuda.synchronize()
    assert rel_err(to_host(y), dy64 * u64 * O.silu_grad(x64)) < tol
    assert rel_err(to_host(y2), dy64 * O.silu(x64)) < tol
    ctx.gelu_forward(code, 0, xd, y)  # empty input
    with pytest.raises(stp.StpError):
        ctx.gelu_forward(code, 12, xd, y)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("seq,mbsz,n,d", [(104, 1, 3, 64), (64, 2, 2, 128), (8, 1, 1, 16)])
def test_rope(ctx, dtype, seq, mbsz, n, d):
    if dtype == "bf16" and d not in (64, 128):
        pytest.skip("bf16 layers take head_dim 64 or 128")
    rng = np.random.default_rng(seq)
    T = seq * mbsz
    for nk in (0, 1):                      # one key / value head per query head, and a single shared one
        nkv = nk or n
        a, ak = n * d, nkv * d
        x = q(rng.standard_normal((T, a + 2 * ak), dtype=np.float32), dtype)
        xd = to_dev(x, dtype)
        wl = synth.Workload("r", 64, n, d, 64, seq, 1, dtype=dtype, rope=True, kv_heads=nk)
        desc = stp.make_desc(wl, mbsz=mbsz)
        for inverse in (False, True):
            buf = xd.clone()
            ctx.rope(desc, buf, inverse=inverse)
            torch.cuda.synchronize()
            got = to_host(buf)
            ref = x.astype(np.float64).copy()
            for b in range(mbsz):
                rows = slice(b * seq, (b + 1) * seq)
                for lo, heads in ((0, n), (a, nkv)):      # the Q heads, then the K heads
                    blk = ref[rows, lo:lo + heads * d].reshape(seq, heads, d)
                    ref[rows, lo:lo + heads * d] = O.rope(blk, 10000.0, inverse).reshape(seq, heads * d)
            assert rel_err(got, ref) < (8e-3 if dtype == "bf16" else 3e-6)
            np.testing.assert_array_equal(got[:, a + ak:], x[:, a + ak:])  # V untouched


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("T,N", [(200, 512), (64, 8), (1000, 1544)])
def test_colsum(ctx, dtype, T, N):
    rng = np.random.default_rng(T)
    x = q(rng.standard_normal((T, N), dtype=np.float32), dtype)
    xd = to_dev(x, dtype)
    out = torch.full((N,), 2.0, dtype=torch.float32, device="cuda")
    ctx.colsum(stp.BF16 if dtype == "bf16" else stp.F32, T, N, xd, 0.125, out, lane=2)
    torch.cuda.synchronize()
    assert rel_err(to_host(out), 2.0 + 0.125 * x.astype(np.float64).sum(0)) < 1e-5


# ------------------------------------------------------------------ stand-alone row softmax
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("rows,n,causal", [(37, 8, False), (64, 1000, False), (130, 2056, False), (24, 4104, False),
                                           (9, 16384, False), (80, 40, True), (300, 1000, True), (4096, 2048, True)])
def test_softmax_forward_backward(ctx, dtype, rows, n, causal):
    rng = np.random.default_rng(rows + n)
    x = q(rng.standard_normal((rows, n), dtype=np.float32) * 3, dtype)
    dy = q(rng.standard_normal((rows, n), dtype=np.float32), dtype)
    xd, dyd = to_dev(x, dtype), to_dev(dy, dtype)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    code = stp.BF16 if dtype == "bf16" else stp.F32
    scale = 0.35
    ctx.softmax_forward(code, rows, n, scale, causal, xd, y)
    ctx.softmax_backward(code, rows, n, scale, y, dyd, dx)
    torch.cuda.synchronize()
    ref = O.softmax_fwd(x.astype(np.float64), scale, causal)
    tol = 8e-3 if dtype == "bf16" else 2e-6
    assert rel_err(to_host(y), ref) < tol
    if causal:      # masked keys get exactly zero
        r = np.arange(rows)[:, None] % n
        assert np.all(to_host(y)[np.arange(n)[None, :] > r] == 0.0)
    # the backward kernel is fed the device's own (rounded) y, and so is the oracle
    refdx = O.softmax_bwd(to_host(y), dy.astype(np.float64), scale)
    assert rel_err(to_host(dx), refdx) < tol


def test_row_kernels_reject_bad_arguments(ctx):
    """Shape, alignment and null-pointer errors of the kernel-level entry points are statuses, raised before any launch."""
    x = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(64 * 64, dtype=torch.float32, device="cuda")
    off = x[1:]                                     # 2 bytes past a 16-byte boundary
    cases = [
        (lambda: ctx.softmax_forward(stp.BF16, 4, 12, 1.0, False, x, x), 2),        # n not a multiple of 8
        (lambda: ctx.softmax_forward(stp.BF16, 4, 16392, 1.0, False, x, x), 2),     # n beyond 16384
        (lambda: ctx.softmax_forward(stp.BF16, 4, 64, 1.0, False, None, x), 1),
        (lambda: ctx.softmax_forward(stp.BF16, 4, 64, 1.0, False, off, x), 3),
        (lambda: ctx.softmax_forward(9, 4, 64, 1.0, False, x, x), 1),
        (lambda: ctx.softmax_backward(stp.BF16, 4, 64, 1.0, x, None, x), 1),
        (lambda: ctx.softmax_backward(stp.BF16, -1, 64, 1.0, x, x, x), 2),
        (lambda: ctx.norm_forward(stp.BF16, stp.NORM_LN, 4, 60, 1e-5, x, x, x, x, f), 2),     # h not a multiple of 8
        (lambda: ctx.norm_forward(stp.BF16, stp.NORM_LN, 4, 8200, 1e-5, x, x, x, x, f), 2),   # h beyond 8192
        (lambda: ctx.norm_forward(stp.BF16, 5, 4, 64, 1e-5, x, x, x, x, f), 1),
        (lambda: ctx.norm_forward(stp.BF16, stp.NORM_LN, 4, 64, 1e-5, x, x, x, off, f), 3),
        (lambda: ctx.norm_forward(stp.BF16, stp.NORM_LN, 4, 64, 1e-5, x, x, x, x, None), 1),
        (lambda: ctx.colsum(stp.BF16, 4, 60, x, 1.0, f), 2),
        (lambda: ctx.colsum(stp.BF16, 4, 64, x, 1.0, f, lane=3), 1),
        (lambda: ctx.colsum(stp.BF16, 4, 64, off, 1.0, f), 3),
        (lambda: ctx.gelu_forward(stp.BF16, 64, off, x), 3),
        (lambda: ctx.gelu_backward(stp.BF16, 64, x, None, x), 1),
    ]
    for i, (call, status) in enumerate(cases):
        with pytest.raises(stp.StpError) as e:
            call()
        assert e.value.status == status, (i, e.value)
    ctx.softmax_forward(stp.BF16, 0, 64, 1.0, False, x, x)      # empty problems are no-ops
    ctx.norm_forward(stp.BF16, stp.NORM_LN, 0, 64, 1e-5, x, x, x, x, f)
    ctx.colsum(stp.BF16, 0, 64, x, 1.0, f)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ attention core
# (dtype, seq, mbsz, query heads, head dim, causal, key / value heads; 0 = one per query head)
ATTN_CASES = [("f32", 128, 1, 4, 64, True, 0), ("f32", 52, 2, 2, 32, False, 0), ("f32", 72, 1, 1, 128, True, 0),
              ("bf16", 128, 1, 2, 128, True, 0), ("bf16", 200, 1, 3, 128, True, 0), ("bf16", 456, 2, 2, 64, True, 0),
              ("bf16", 328, 1, 2, 64, False, 0), ("bf16", 1000, 1, 1, 128, False, 0), ("bf16", 8, 1, 1, 128, True, 0),
              # longer than one chunk of keys / queries: the chunk partials and combine kernels
              ("bf16", 2568, 1, 1, 128, True, 0), ("bf16", 1288, 2, 2, 64, False, 0), ("bf16", 2104, 1, 1, 64, True, 0),
              ("bf16", 4360, 1, 1, 128, True, 0),
              # grouped-query attention: groups of 2, 3 and 5 query heads per key / value head
              ("f32", 96, 2, 4, 32, True, 2), ("bf16", 264, 1, 6, 128, True, 2), ("bf16", 520, 2, 4, 64, False, 2),
              ("bf16", 1160, 1, 5, 128, True, 1),
              # 7 query heads over one key / value head (the 56 / 8-head model of Section 5.1 at TP = 8)
              ("bf16", 904, 1, 7, 128, True, 1), ("f32", 40, 1, 7, 16, True, 1)]


@pytest.mark.parametrize("dtype,seq,mbsz,n,d,causal,nk", ATTN_CASES)
def test_attention_forward_backward(ctx, dtype, seq, mbsz, n, d, causal, nk):
    rng = np.random.default_rng(seq * 3 + d)
    nkv = nk or n
    a, ak, T = n * d, nkv * d, seq * mbsz
    qkv = q(rng.standard_normal((T, a + 2 * ak), dtype=np.float32), dtype)
    dctx = q(rng.standard_normal((T, a), dtype=np.float32), dtype)
    qkvd, dctxd = to_dev(qkv, dtype), to_dev(dctx, dtype)
    wl = synth.Workload("a", 64, n, d, 64, seq, 1, dtype=dtype, causal=causal, kv_heads=nk)
    desc = stp.make_desc(wl, mbsz=mbsz)
    out = torch.zeros((T, a), dtype=qkvd.dtype, device="cuda")
    lse = torch.zeros((mbsz, n, seq), dtype=torch.float32, device="cuda")
    delta = torch.zeros_like(lse)
    dqkv = torch.zeros_like(qkvd)
    ctx.attention_forward(desc, qkvd, out, lse)
    ctx.attention_backward(desc, qkvd, out, lse, dctxd, delta, dqkv)
    torch.cuda.synchronize()
    tol = 1e-2 if dtype == "bf16" else 3e-6
    q64 = qkv.astype(np.float64)
    got_o, got_d, got_l = to_host(out), to_host(dqkv), to_host(lse)
    for b in range(mbsz):
        rows = slice(b * seq, (b + 1) * seq)
        Q = q64[rows, :a].reshape(seq, n, d)
        K, V = (q64[rows, a + i * ak:a + (i + 1) * ak].reshape(seq, nkv, d) for i in range(2))
        ref = O.attention_fwd(Q, K, V, causal)
        assert rel_err(got_o[rows], ref.reshape(seq, a)) < tol
        dq, dk, dv = O.attention_bwd(Q, K, V, dctx.astype(np.float64)[rows].reshape(seq, n, d), causal)
        ref_d = np.concatenate([dq.reshape(seq, a), dk.reshape(seq, ak), dv.reshape(seq, ak)], axis=1)
        for name, sl in (("q", slice(0, a)), ("k", slice(a, a + ak)), ("v", slice(a + ak, a + 2 * ak))):
            assert rel_err(got_d[rows, sl], ref_d[:, sl]) < tol, name
        for hd in range(n):  # log-sum-exp of the scaled, masked scores
            S = Q[:, hd] @ K[:, hd // (n // nkv)].T / math.sqrt(d)
            if causal:
                S = np.where(np.tril(np.ones((seq, seq), bool)), S, -np.inf)
            mx = S.max(1)
            ref_l = mx + np.log(np.exp(S - mx[:, None]).sum(1))
            assert np.max(np.abs(got_l[b, hd] - ref_l)) < (2e-2 if dtype == "bf16" else 1e-5)
