"""Shared plumbing of the GPU parity tests: moves the seeded host tensors to the device
in the workload's storage type, owns stashes / gradient buffers, and runs the oracle on
the very same (already rounded) values."""
from __future__ import annotations

import ctypes as C
from dataclasses import replace

import numpy as np
import torch

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import synth
from oracle import stp_oracle as O


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 host values -> device tensor of the storage type (bf16 by bit pattern: no second rounding)."""
    if dtype == "bf16":
        bits = synth.to_bf16_bits(x).view(np.int16)
        return torch.from_numpy(bits.copy()).cuda().view(torch.bfloat16).reshape(x.shape)
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max|got - ref| / max|ref| (the tolerance definition used for every parity check)."""
    den = float(np.max(np.abs(ref)))
    return float(np.max(np.abs(np.asarray(got, np.float64) - ref))) / (den if den > 0 else 1.0)


# half a unit in the last place of a stored value, relative to the value (24 / 8 significant bits): the one
# rounding of the sum branch + residual
STORE_ULP = {"f32": 2.0 ** -24, "bf16": 2.0 ** -8}


def branch_err(got, got_resid, ref, ref_resid, coeff: float, dtype: str) -> float:
    """Parity of the computed branch of a residual-carrying output (Eq. 1: out = branch + X/t; Eq. 2:
    dX = norm_bwd(..) + dY), which max|got - ref| / max|ref| dilutes when the residual dominates the output.
    Each side has its own residual input subtracted (the path's is the value it stored, already rounded; the
    oracle's is its own), so what is compared is what the unit computed.  The bound is the parity tolerance
    relative to max|branch| plus the one rounding of the stored sum, half a unit in the last place of max|out|.
    Returns error / bound: below 1 passes."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    b_got = got - coeff * np.asarray(got_resid, np.float64).reshape(got.shape)
    b_ref = ref - coeff * np.asarray(ref_resid, np.float64).reshape(ref.shape)
    bound = TOL[dtype] * float(np.max(np.abs(b_ref))) + STORE_ULP[dtype] * float(np.max(np.abs(ref)))
    return float(np.max(np.abs(b_got - b_ref))) / (bound if bound > 0 else 1.0)


def oracle_cfg(wl: synth.Workload) -> O.LayerCfg:
    return O.LayerCfg(hidden=wl.hidden, heads_local=wl.heads_local, head_dim=wl.head_dim, ffn_local=wl.ffn_local,
                      tp=wl.tp, norm=wl.norm, act=wl.act, causal=wl.causal, rope=wl.rope, has_bias=wl.has_bias,
                      eps=wl.eps, rope_base=wl.rope_base, kv_heads_local=wl.kv_heads)


TOL = {"f32": 1e-5, "bf16": 2e-2}


class LayerOnDevice:
    """One layer's weights, fp32 gradient accumulators and per-microbatch stashes on the GPU."""

    def __init__(self, ctx: stp.Context, wl: synth.Workload, seed: int, layer: int = 0, n_mb: int = 1, mbsz: int = 1):
        self.ctx, self.wl, self.mbsz = ctx, wl, mbsz
        self.desc = stp.make_desc(wl, mbsz=mbsz)
        self.tdtype = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        self.w_host = synth.make_weights(wl, seed, layer)
        self.w_dev = {k: to_dev(v, wl.dtype) for k, v in self.w_host.items()}
        self.g_dev = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in self.w_host.items()}
        self.w = stp.Weights(**{k: v.data_ptr() for k, v in self.w_dev.items()})
        self.g = stp.WGrads(**{k: v.data_ptr() for k, v in self.g_dev.items()})
        # Every accumulator goes to exactly one unit.  The row-parallel bias gradients b_o / b_fc2 can be filled by
        # the W units (tables g_b / g) or ride in the norm backward of the Pre-* B units (tables g_b_bias / g_w_nobias).
        ptr = {k: v.data_ptr() for k, v in self.g_dev.items()}
        norm_keys = [k for k in ptr if k.startswith("norm")]
        self.g_b = stp.WGrads(**{k: ptr[k] for k in norm_keys})
        self.g_b_bias = stp.WGrads(**{k: ptr[k] for k in norm_keys + [k for k in ("b_o", "b_fc2") if k in ptr]})
        self.g_w_nobias = stp.WGrads(**{k: v for k, v in ptr.items() if k not in ("b_o", "b_fc2")})
        nbytes = ctx.stash_bytes(self.desc)
        self.stash_mem = [torch.zeros(nbytes, dtype=torch.uint8, device="cuda") for _ in range(n_mb)]
        self.stash = [stp.Stash(base=m.data_ptr(), bytes=nbytes) for m in self.stash_mem]
        ctx.ensure_workspace([self.desc])

    def field(self, name: str, mb: int = 0) -> torch.Tensor:
        """View of a stash field as a typed tensor."""
        off, n = self.ctx.stash_field(self.desc, name)
        raw = self.stash_mem[mb][off:off + n]
        if name in ("STATS1", "STATS2", "LSE", "DELTA"):
            return raw.view(torch.float32)
        return raw.view(self.tdtype)

    def new_act(self) -> torch.Tensor:
        return torch.empty((self.wl.seq * self.mbsz, self.wl.hidden), dtype=self.tdtype, device="cuda")

    def w64(self):
        return {k: v.astype(np.float64) for k, v in self.w_host.items()}


def gpu_layer_pass(ctx, lay: LayerOnDevice, X: torch.Tensor, dO: torch.Tensor, mb: int = 0, stream=None,
                   bias_in_b: bool = False):
    """F units, then B units, then W units of one rank with identity at the AR points.  bias_in_b: the Pre-* B units
    fill b_o / b_fc2 (as stp_braid_step wires it) instead of the W units."""
    d, w, st = lay.desc, lay.w, lay.stash[mb]
    g_b, g_w = (lay.g_b_bias, lay.g_w_nobias) if bias_in_b else (lay.g_b, lay.g)
    out = {k: lay.new_act() for k in ("x_attn", "x_out", "dz", "dx_attn", "dx_ln", "dx")}
    ctx.forward_unit(d, stp.PRE_ATTN, w, st, x_in=X, stream=stream)
    ctx.forward_unit(d, stp.ATTN, w, st, x_resid=X, y_out=out["x_attn"], stream=stream)
    ctx.forward_unit(d, stp.PRE_MLP, w, st, x_in=out["x_attn"], stream=stream)
    ctx.forward_unit(d, stp.MLP, w, st, x_resid=out["x_attn"], y_out=out["x_out"], stream=stream)
    ctx.backward_input_unit(d, stp.MLP, w, st, dy=dO, dx=out["dz"], stream=stream)
    ctx.backward_input_unit(d, stp.PRE_MLP, w, st, x_in=out["x_attn"], dy=out["dz"], d_resid=dO, dx=out["dx_attn"],
                            wgrads=g_b, stream=stream)
    ctx.backward_input_unit(d, stp.ATTN, w, st, dy=out["dx_attn"], dx=out["dx_ln"], stream=stream)
    ctx.backward_input_unit(d, stp.PRE_ATTN, w, st, x_in=X, dy=out["dx_ln"], d_resid=out["dx_attn"], dx=out["dx"],
                            wgrads=g_b, stream=stream)
    ctx.backward_weight_unit(d, stp.MLP, st, dO, g_w, stream=stream)
    ctx.backward_weight_unit(d, stp.ATTN, st, out["dx_attn"], g_w, stream=stream)
    return out


def oracle_layer_pass(cfg: O.LayerCfg, W: dict, X: np.ndarray, dO: np.ndarray, grads: dict = None):
    """The same sequence in the fp64 oracle; returns activations, stash and gradients."""
    st, g = {}, ({} if grads is None else grads)
    r = {}
    O.forward_unit(cfg, O.PRE_ATTN, W, st, x_in=X)
    r["x_attn"] = O.forward_unit(cfg, O.ATTN, W, st, x_resid=X)
    O.forward_unit(cfg, O.PRE_MLP, W, st, x_in=r["x_attn"])
    r["x_out"] = O.forward_unit(cfg, O.MLP, W, st, x_resid=r["x_attn"])
    r["dz"] = O.backward_input_unit(cfg, O.MLP, W, st, dO)
    r["dx_attn"] = O.backward_input_unit(cfg, O.PRE_MLP, W, st, r["dz"], d_resid=dO, grads=g)
    r["dx_ln"] = O.backward_input_unit(cfg, O.ATTN, W, st, r["dx_attn"])
    r["dx"] = O.backward_input_unit(cfg, O.PRE_ATTN, W, st, r["dx_ln"], d_resid=r["dx_attn"], grads=g)
    O.backward_weight_unit(cfg, O.MLP, st, dO, g)
    O.backward_weight_unit(cfg, O.ATTN, st, r["dx_attn"], g)
    return r, st, g
