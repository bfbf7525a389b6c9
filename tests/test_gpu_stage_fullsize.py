"""One pipeline stage at full size through the whole braided sequence on three streams: 4 GPT-7B TP=8 layers
at seq 4096 with 8 microbatches (the first and last microbatch followed through all four layers by the fp64
oracle: stage output and input gradient, element by element), and the heterogeneous ViT + LM stage."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import synth
from paper_2510_27257_amd.stage import StageOnDevice, stage_sequence
from oracle import stp_oracle as O
from harness import TOL, oracle_cfg, rel_err, to_host


def test_four_layer_stage_sequence_matches_oracle():
    wl = synth.WORKLOADS["gpt7b_tp8_s4096"]
    L, n_mb = 4, 8
    ctx = stp.Context(0)
    stg = StageOnDevice(ctx, [wl] * L, n_mb, seed=0)
    assert stg.tuned_objective == "stage" and stg.tuned == [wl.name]      # the table measured on a stage's sequence
    stg.load_inputs()
    sF, sB, sW = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    ctx.braid_reset()
    for step in stage_sequence(L, n_mb):
        ctx.braid_step(stg.stage, step, sF, sB, sW)
    torch.cuda.synchronize()
    print("GPU sequence done; running the oracle for microbatches 0 and 7", flush=True)
    cfg = oracle_cfg(wl)
    errs = {}
    for mb in (0, n_mb - 1):
        x = synth.make_activation(wl, 0, f"x.mb{mb}").astype(np.float64)
        stashes = []
        for l in range(L):
            W = {k: v.astype(np.float64) for k, v in stg.w_host[l].items()}
            st = {}
            O.forward_unit(cfg, O.PRE_ATTN, W, st, x_in=x)
            xa = O.forward_unit(cfg, O.ATTN, W, st, x_resid=x)
            O.forward_unit(cfg, O.PRE_MLP, W, st, x_in=xa)
            x = O.forward_unit(cfg, O.MLP, W, st, x_resid=xa)
            stashes.append(st)
        errs[f"out.mb{mb}"] = rel_err(to_host(stg.act_slot(L, mb)), x)
        dy = synth.make_activation(wl, 0, f"dy.mb{mb}").astype(np.float64)
        for l in reversed(range(L)):
            W = {k: v.astype(np.float64) for k, v in stg.w_host[l].items()}
            st = stashes[l]
            dz = O.backward_input_unit(cfg, O.MLP, W, st, dy)
            dxa = O.backward_input_unit(cfg, O.PRE_MLP, W, st, dz, d_resid=dy)
            dxl = O.backward_input_unit(cfg, O.ATTN, W, st, dxa)
            dy = O.backward_input_unit(cfg, O.PRE_ATTN, W, st, dxl, d_resid=dxa)
            stashes[l] = None
        errs[f"dx.mb{mb}"] = rel_err(to_host(stg.grad_slot(0, mb)), dy)
        print(errs, flush=True)
    ctx.close()
    bad = {k: v for k, v in errs.items() if not v < TOL["bf16"]}
    assert not bad, bad


def test_heterogeneous_stage_sequence_matches_oracle():
    """A stage of two full-size ViT layers (bidirectional, 1024 tokens) followed, after a chain break, by two
    GPT-7B TP=8 layers at seq 4096 (the multimodal case of Section 4.1), 8 microbatches through the braided
    sequence on three streams.  The oracle follows one microbatch through each chain, forward and backward."""
    vit, lm = synth.WORKLOADS["vit"], synth.WORKLOADS["gpt7b_tp8_s4096"]
    layers, cb, n_mb = [vit, vit, lm, lm], [0, 0, 1, 0, 0], 8
    L = len(layers)
    ctx = stp.Context(0)
    stg = StageOnDevice(ctx, layers, n_mb, seed=0, chain_break=cb)
    stg.load_inputs()
    sF, sB, sW = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    ctx.braid_reset()
    for step in stage_sequence(L, n_mb):
        ctx.braid_step(stg.stage, step, sF, sB, sW)
    torch.cuda.synchronize()
    print("GPU sequence done; running the oracle for one microbatch per chain", flush=True)
    errs = {}
    for ci, ((first, last), mb) in enumerate(zip(stg.chains(), (n_mb - 1, 0))):
        x = synth.make_activation(layers[first], 0, f"c{ci}.x.mb{mb}").astype(np.float64)
        stashes = {}
        for l in range(first, last + 1):
            cfg, W = oracle_cfg(layers[l]), {k: v.astype(np.float64) for k, v in stg.w_host[l].items()}
            st = {}
            O.forward_unit(cfg, O.PRE_ATTN, W, st, x_in=x)
            xa = O.forward_unit(cfg, O.ATTN, W, st, x_resid=x)
            O.forward_unit(cfg, O.PRE_MLP, W, st, x_in=xa)
            x = O.forward_unit(cfg, O.MLP, W, st, x_resid=xa)
            stashes[l] = st
        errs[f"chain{ci}.out.mb{mb}"] = rel_err(to_host(stg.chain_output(last, mb)), x)
        dy = synth.make_activation(layers[last], 0, f"c{ci}.dy.mb{mb}").astype(np.float64)
        for l in range(last, first - 1, -1):
            cfg, W = oracle_cfg(layers[l]), {k: v.astype(np.float64) for k, v in stg.w_host[l].items()}
            st = stashes.pop(l)
            dz = O.backward_input_unit(cfg, O.MLP, W, st, dy)
            dxa = O.backward_input_unit(cfg, O.PRE_MLP, W, st, dz, d_resid=dy)
            dxl = O.backward_input_unit(cfg, O.ATTN, W, st, dxa)
            dy = O.backward_input_unit(cfg, O.PRE_ATTN, W, st, dxl, d_resid=dxa)
        errs[f"chain{ci}.dx.mb{mb}"] = rel_err(to_host(stg.grad_slot(first, mb)), dy)
        print(errs, flush=True)
    ctx.close()
    bad = {k: v for k, v in errs.items() if not v < TOL["bf16"]}
    assert not bad, bad
