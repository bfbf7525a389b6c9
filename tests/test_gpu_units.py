"""Per-unit parity of the F / B / W units against the fp64 oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import synth
from paper_2510_27257_amd.synth import Workload
from oracle import stp_oracle as O
from harness import (LayerOnDevice, TOL, branch_err, gpu_layer_pass, oracle_cfg, oracle_layer_pass, rel_err, to_dev, to_host)

# sizes the oracle finishes in seconds that still span several 128/256 tiles and leave ragged tails
CASES = {
    "tiny_fp32": synth.WORKLOADS["tiny"],
    "gpt_bf16": Workload("gpt_bf16", 512, 2, 128, 1032, 328, 8),
    "llama_bf16": Workload("llama_bf16", 640, 3, 128, 712, 264, 4, norm="rms", act="swiglu", rope=True, has_bias=False),
    "vit_bf16": Workload("vit_bf16", 256, 4, 64, 520, 200, 1, causal=False),
    "llama_fp32": Workload("llama_fp32", 128, 2, 32, 200, 72, 4, dtype="f32", norm="rms", act="swiglu", rope=True,
                           has_bias=False),
    "gpt_fp32_tp2": Workload("gpt_fp32_tp2", 64, 2, 16, 96, 40, 2, dtype="f32"),
    # grouped-query attention: 6 query heads over 2 key / value heads (bf16), 4 over 1 (fp32, with biases)
    "gqa_bf16": Workload("gqa_bf16", 512, 6, 128, 712, 264, 4, norm="rms", act="swiglu", rope=True, has_bias=False, kv_heads=2),
    "gqa_fp32": Workload("gqa_fp32", 96, 4, 32, 136, 56, 8, dtype="f32", rope=True, kv_heads=1),
}


@pytest.fixture(scope="module")
def ctx():
    c = stp.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


@pytest.mark.parametrize("bias_in_b", [False, True], ids=["bias_grads_in_W", "bias_grads_in_PreB"])
@pytest.mark.parametrize("name", list(CASES))
def test_units_match_oracle(ctx, name, bias_in_b):
    """Every unit output, stash field and weight gradient against the oracle.  The gradients of the row-parallel
    biases (b_o, b_fc2) are (1/t) of the column sum of the Attn / MLP unit's upstream gradient: the W units
    compute them when handed the accumulators, and so do the Pre-Attn-B / Pre-MLP-B units (which read that
    gradient on their residual path, Eq. 2); both routes are run."""
    wl = CASES[name]
    if bias_in_b and not wl.has_bias:
        pytest.skip("no biases in this layer")
    tol = TOL[wl.dtype]
    lay = LayerOnDevice(ctx, wl, seed=0)
    X = synth.make_activation(wl, 0, "x.mb0")
    dO = synth.make_activation(wl, 0, "dy.mb0")
    got = gpu_layer_pass(ctx, lay, to_dev(X, wl.dtype), to_dev(dO, wl.dtype), bias_in_b=bias_in_b)
    torch.cuda.synchronize()
    ref, st, g = oracle_layer_pass(oracle_cfg(wl), lay.w64(), X.astype(np.float64), dO.astype(np.float64))
    T, a = wl.seq, wl.attn_local
    errs = {}
    for k in ("x_attn", "x_out", "dz", "dx_attn", "dx_ln", "dx"):
        errs[k] = rel_err(to_host(got[k]), ref[k])
    qkv_ref = np.concatenate([st[k].reshape(T, -1) for k in ("q", "k", "v")], axis=1)
    stash_checks = {"X_LN": st["x_ln"], "QKV": qkv_ref, "CTX": st["ctx"], "Z_LN": st["z_ln"], "H": st["h"],
                    "G": st["g"], "DH": st["dh"], "DQKV": st["dqkv"]}
    if wl.act == "swiglu":
        stash_checks.update(HU=st["hu"], DHU=st["dhu"])
    for f, r in stash_checks.items():
        errs["stash." + f] = rel_err(to_host(lay.field(f)).reshape(r.shape), r)
    assert set(g) == set(lay.g_dev)
    for k, r in g.items():
        errs["grad." + k] = rel_err(to_host(lay.g_dev[k]), r)
    bad = {k: v for k, v in errs.items() if not v < tol}
    assert not bad, f"{name}: over tolerance {tol}: {bad}\nall: {errs}"
    # the residual-carrying outputs once more with the residual taken off, so that an error of the computed
    # branch is not measured against the (larger) residual
    X64, dO64 = X.astype(np.float64), dO.astype(np.float64)
    branch = {"x_attn": branch_err(to_host(got["x_attn"]), X64, ref["x_attn"], X64, 1.0 / wl.tp, wl.dtype),
              "x_out": branch_err(to_host(got["x_out"]), to_host(got["x_attn"]), ref["x_out"], ref["x_attn"], 1.0 / wl.tp, wl.dtype),
              "dx_attn": branch_err(to_host(got["dx_attn"]), dO64, ref["dx_attn"], dO64, 1.0, wl.dtype),
              "dx": branch_err(to_host(got["dx"]), to_host(got["dx_attn"]), ref["dx"], ref["dx_attn"], 1.0, wl.dtype)}
    bad = {k: v for k, v in branch.items() if not v < 1.0}
    assert not bad, f"{name}: computed branch over its bound (error / bound): {bad}\nall: {branch}"


@pytest.mark.parametrize("name", ["gpt_bf16", "gpt_fp32_tp2"])
def test_units_with_two_sequences_per_microbatch(ctx, name):
    """mbsz = 2: tokens = 2 * seq; attention must not mix the two sequences, everything else is row-wise."""
    wl = CASES[name]
    tol = TOL[wl.dtype]
    lay = LayerOnDevice(ctx, wl, seed=4, mbsz=2)
    Xs = [synth.make_activation(wl, 4, f"x.s{i}") for i in range(2)]
    dOs = [synth.make_activation(wl, 4, f"dy.s{i}") for i in range(2)]
    got = gpu_layer_pass(ctx, lay, to_dev(np.concatenate(Xs), wl.dtype), to_dev(np.concatenate(dOs), wl.dtype))
    torch.cuda.synchronize()
    g_ref, outs, dxs = {}, [], []
    for X, dO in zip(Xs, dOs):   # the oracle sees the two sequences as two microbatches of one sequence
        ref, _, _ = oracle_layer_pass(oracle_cfg(wl), lay.w64(), X.astype(np.float64), dO.astype(np.float64), grads=g_ref)
        outs.append(ref["x_out"]); dxs.append(ref["dx"])
    assert rel_err(to_host(got["x_out"]), np.concatenate(outs)) < tol
    assert rel_err(to_host(got["dx"]), np.concatenate(dxs)) < tol
    for k, r in g_ref.items():
        assert rel_err(to_host(lay.g_dev[k]), r) < tol, k


def test_weight_grads_accumulate_across_microbatches(ctx):
    wl = CASES["gpt_fp32_tp2"]
    lay = LayerOnDevice(ctx, wl, seed=3, n_mb=2)
    g_ref = {}
    for mb in range(2):
        X = synth.make_activation(wl, 3, f"x.mb{mb}")
        dO = synth.make_activation(wl, 3, f"dy.mb{mb}")
        gpu_layer_pass(ctx, lay, to_dev(X, wl.dtype), to_dev(dO, wl.dtype), mb=mb)
        oracle_layer_pass(oracle_cfg(wl), lay.w64(), X.astype(np.float64), dO.astype(np.float64), grads=g_ref)
    torch.cuda.synchronize()
    for k, r in g_ref.items():
        assert rel_err(to_host(lay.g_dev[k]), r) < 1e-5, k


@pytest.mark.parametrize("t", [2, 4])
def test_tp_sum_on_gpu_reproduces_unsharded_oracle(ctx, t):
    """Eq. 1-2 on the device: run all t ranks one after the other, sum their partials at the four
    AR points, and compare with the oracle's UNSHARDED layer (x_out, dX)."""
    full = Workload("full", 64, 4, 16, 128, 48, 1, dtype="f32")
    Wfull = {k: v.astype(np.float64) for k, v in synth.make_weights(full, 11).items()}
    X = synth.make_activation(full, 11, "x")
    dO = synth.make_activation(full, 11, "dy")
    ref_out, ref_st = O.layer_forward_all_ranks(oracle_cfg(full), [Wfull], X.astype(np.float64))
    ref_dx, _ = O.layer_backward_all_ranks(oracle_cfg(full), [Wfull], ref_st, dO.astype(np.float64))

    shard_wl = Workload("shard", 64, 4 // t, 16, 128 // t, 48, t, dtype="f32")
    lays = []
    for r in range(t):
        lay = LayerOnDevice(ctx, shard_wl, seed=0)
        _, ws = O.shard_weights(oracle_cfg(full), Wfull, t, r)
        for k, v in ws.items():
            lay.w_dev[k].copy_(torch.from_numpy(np.ascontiguousarray(v, np.float32)))
        lays.append(lay)
    Xd, dOd = to_dev(X, "f32"), to_dev(dO, "f32")
    d = lays[0].desc

    def all_ranks(fn):
        parts = []
        for lay in lays:
            buf = lay.new_act()
            fn(lay, buf)
            parts.append(buf)
        return torch.stack(parts).sum(0)          # the All-Reduce the boundary stands for

    for lay in lays:
        ctx.forward_unit(d, stp.PRE_ATTN, lay.w, lay.stash[0], x_in=Xd)
    x_attn = all_ranks(lambda lay, y: ctx.forward_unit(d, stp.ATTN, lay.w, lay.stash[0], x_resid=Xd, y_out=y))
    for lay in lays:
        ctx.forward_unit(d, stp.PRE_MLP, lay.w, lay.stash[0], x_in=x_attn)
    x_out = all_ranks(lambda lay, y: ctx.forward_unit(d, stp.MLP, lay.w, lay.stash[0], x_resid=x_attn, y_out=y))
    dz = all_ranks(lambda lay, y: ctx.backward_input_unit(d, stp.MLP, lay.w, lay.stash[0], dy=dOd, dx=y))
    dxa = lays[0].new_act()
    ctx.backward_input_unit(d, stp.PRE_MLP, lays[0].w, lays[0].stash[0], x_in=x_attn, dy=dz, d_resid=dOd, dx=dxa)
    dxl = all_ranks(lambda lay, y: ctx.backward_input_unit(d, stp.ATTN, lay.w, lay.stash[0], dy=dxa, dx=y))
    dx = lays[0].new_act()
    ctx.backward_input_unit(d, stp.PRE_ATTN, lays[0].w, lays[0].stash[0], x_in=Xd, dy=dxl, d_resid=dxa, dx=dx)
    torch.cuda.synchronize()
    assert rel_err(to_host(x_out), ref_out) < 1e-5
    assert rel_err(to_host(dx), ref_dx) < 1e-5


def test_units_reject_bad_arguments(ctx):
    wl = CASES["gpt_fp32_tp2"]
    lay = LayerOnDevice(ctx, wl, seed=0)
    X = to_dev(synth.make_activation(wl, 0, "x"), "f32")
    with pytest.raises(stp.StpError) as e:
        ctx.forward_unit(lay.desc, stp.PRE_ATTN, lay.w, lay.stash[0], x_in=None)
    assert e.value.status == 1
    with pytest.raises(stp.StpError) as e:
        ctx.forward_unit(lay.desc, stp.PRE_ATTN, lay.w, lay.stash[0], x_in=X.data_ptr() + 4)
    assert e.value.status == 3
    small = stp.Stash(base=lay.stash[0].base, bytes=1024)
    with pytest.raises(stp.StpError) as e:
        ctx.forward_unit(lay.desc, stp.PRE_ATTN, lay.w, small, x_in=X)
    assert e.value.status == 4
    with pytest.raises(stp.StpError) as e:
        ctx.forward_unit(lay.desc, 9, lay.w, lay.stash[0], x_in=X)
    assert e.value.status == 1
    with pytest.raises(stp.StpError) as e:
        ctx.backward_weight_unit(lay.desc, stp.PRE_MLP, lay.stash[0], X, lay.g)
    assert e.value.status == 1
    bad = stp.make_desc(wl)
    bad.hidden = 60
    with pytest.raises(stp.StpError) as e:
        ctx.forward_unit(bad, stp.PRE_ATTN, lay.w, lay.stash[0], x_in=X)
    assert e.value.status == 2
