"""Parity at the full benchmark sizes, in the launch configuration bench.py times: one braided
block F(mb1) | B+W(mb0) on three streams, every output tensor compared with the fp64 oracle
element by element (the numpy oracle finishes a full-size layer-microbatch in seconds)."""
import os

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import synth
from paper_2510_27257_amd.binding import OP_BW
from paper_2510_27257_amd.stage import StageOnDevice, backward_ops, braid, forward_ops
from oracle import stp_oracle as O
from harness import TOL, branch_err, oracle_cfg, oracle_layer_pass, rel_err, to_host


OBSERVED = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "fullsize_bf16_observed_errors.txt")


def observed_errors(name):
    """Per-tensor errors this block showed when the table was written (a drift alarm beside the tolerance)."""
    out = {}
    if os.path.exists(OBSERVED):
        for line in open(OBSERVED):
            parts = line.split()
            if len(parts) == 3 and parts[0] == name:
                out[parts[1]] = float(parts[2])
    return out


# the benchmark configurations, then the shards of the two language models of the model table of Section 5.1 at
# sequence lengths of their throughput rows: 10 / 2, 5 / 1 (12.1B at TP 4 / 8) and 7 / 1 (26.3B at TP 8) query /
# key-value heads on the rank
@pytest.mark.parametrize("name", ["gpt7b_tp8", "llama13b_tp4", "vit", "gqa12b_tp4", "gqa12b_tp4_s6144", "gqa12b_tp8_s3072",
                                  "gqa26b_tp8", "gqa26b_tp8_s2048"])
def test_full_size_braided_block_matches_oracle(name):
    wl = synth.WORKLOADS[name]
    tol = TOL[wl.dtype]
    ctx = stp.Context(0)
    stg = StageOnDevice(ctx, [wl], n_mb=2, seed=0)
    assert stg.tuned_objective == "block"         # the launch configuration the benchmark times: its tile preferences
    stg.load_inputs()
    sF, sB, sW = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    ctx.braid_reset()
    ctx.braid_step(stg.stage, forward_ops(1, 0), sF, sB, sW)
    ctx.braid_step(stg.stage, braid(forward_ops(1, 1), backward_ops(1, 0, OP_BW)), sF, sB, sW)
    torch.cuda.synchronize()
    print(f"[{name}] GPU done; running the fp64 oracle", flush=True)
    cfg = oracle_cfg(wl)
    W = {k: v.astype(np.float64) for k, v in stg.w_host[0].items()}
    X0 = synth.make_activation(wl, 0, "x.mb0").astype(np.float64)
    dO = synth.make_activation(wl, 0, "dy.mb0").astype(np.float64)
    ref, st, g = oracle_layer_pass(cfg, W, X0, dO)
    errs = {"x_out.mb0": rel_err(to_host(stg.act_slot(1, 0)), ref["x_out"]),
            "dx.mb0": rel_err(to_host(stg.grad_slot(0, 0)), ref["dx"]),
            "x_attn.mb0": rel_err(to_host(stg.field(0, 0, "X_ATTN")).reshape(ref["x_attn"].shape), ref["x_attn"]),
            "dx_attn.mb0": rel_err(to_host(stg.field(0, 0, "DX_ATTN")).reshape(ref["dx_attn"].shape), ref["dx_attn"]),
            "ctx.mb0": rel_err(to_host(stg.field(0, 0, "CTX")).reshape(st["ctx"].shape), st["ctx"]),
            "dqkv.mb0": rel_err(to_host(stg.field(0, 0, "DQKV")).reshape(st["dqkv"].shape), st["dqkv"])}
    for k, r in g.items():
        errs["grad." + k] = rel_err(to_host(stg.g_dev[0][k]), r)
    # the residual-carrying outputs of Eq. 1 / Eq. 2 with the residual taken off (error / bound, below 1 passes)
    xa_gpu = to_host(stg.field(0, 0, "X_ATTN")).reshape(ref["x_attn"].shape)
    dxa_gpu = to_host(stg.field(0, 0, "DX_ATTN")).reshape(ref["dx_attn"].shape)
    branch = {"x_attn.mb0": branch_err(xa_gpu, X0, ref["x_attn"], X0, 1.0 / wl.tp, wl.dtype),
              "x_out.mb0": branch_err(to_host(stg.act_slot(1, 0)), xa_gpu, ref["x_out"], ref["x_attn"], 1.0 / wl.tp, wl.dtype),
              "dx_attn.mb0": branch_err(dxa_gpu, dO, ref["dx_attn"], dO, 1.0, wl.dtype),
              "dx.mb0": branch_err(to_host(stg.grad_slot(0, 0)), dxa_gpu, ref["dx"], ref["dx_attn"], 1.0, wl.dtype)}
    del ref, st, g
    # the forward half of the block (microbatch 1)
    X1 = synth.make_activation(wl, 0, "x.mb1").astype(np.float64)
    st1 = {}
    O.forward_unit(cfg, O.PRE_ATTN, W, st1, x_in=X1)
    xa = O.forward_unit(cfg, O.ATTN, W, st1, x_resid=X1)
    O.forward_unit(cfg, O.PRE_MLP, W, st1, x_in=xa)
    out1 = O.forward_unit(cfg, O.MLP, W, st1, x_resid=xa)
    errs["x_out.mb1"] = rel_err(to_host(stg.act_slot(1, 1)), out1)
    ctx.close()
    print(f"[{name}] {errs}", flush=True)
    print(f"[{name}] computed branches, error / bound: {branch}", flush=True)
    bad = {k: v for k, v in errs.items() if not v < tol}
    assert not bad, f"{name}: over tolerance {tol}: {bad}"
    bad = {k: v for k, v in branch.items() if not v < 1.0}
    assert not bad, f"{name}: computed branch over its bound: {bad}"
    record = os.environ.get("STP_RECORD_ERRORS")
    if record:
        with open(record, "a") as f:
            for k, v in errs.items():
                f.write(f"{name} {k} {v:.4e}\n")
        return
    seen = observed_errors(name)
    drift = {k: (v, seen[k]) for k, v in errs.items() if k in seen and not v < 1.5 * seen[k] + 1e-6}
    assert not drift, f"{name}: error (now, when the table was written) grew by more than half: {drift}"
