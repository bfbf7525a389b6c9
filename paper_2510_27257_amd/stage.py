"""Device-side container for one pipeline stage's model chunk (Section 4.2): per-layer weights
and gradient accumulators, per (layer, microbatch) stashes, the activation / gradient slots
between layers, and the ctypes tables stp_braid_step reads.  Also the canonical op lists of the
braided blocks.  Argument marshalling and torch allocations only: no arithmetic of the method."""
from __future__ import annotations

import ctypes as C
from typing import List, Optional, Sequence

import torch

from . import binding as B
from . import synth


def _to_dev(x, dtype: str) -> torch.Tensor:
    import numpy as np
    if dtype == "bf16":
        bits = synth.to_bf16_bits(x).view(np.int16)
        return torch.from_numpy(bits.copy()).cuda().view(torch.bfloat16).reshape(x.shape)
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()


class StageOnDevice:
    def __init__(self, ctx: B.Context, layers: Sequence[synth.Workload], n_mb: int, seed: int = 0,
                 chain_break: Optional[Sequence[int]] = None, tuned_tiles=True):
        self.ctx, self.layers, self.n_mb, self.seed = ctx, list(layers), n_mb, seed
        L = len(self.layers)
        # measured GEMM tile preferences for these layers' GEMMs beside other streams, where the package has some
        # (they change the time of a step, never its results).  tuned_tiles: False leaves the context's hints as
        # they are; "block" / "stage" names the objective they were measured for; True takes "block" for a
        # single layer (its braided block issued back to back) and "stage" for several (a stage's sequence of
        # steps).  A context holds the preferences of the stage built last.
        from . import tune
        self.tuned, self.tuned_objective, self.n_tile_hints = [], None, 0
        if tuned_tiles:
            self.tuned_objective = tuned_tiles if isinstance(tuned_tiles, str) else ("block" if L == 1 else "stage")
            ctx.gemm_tile_hints_clear()
            self.tuned = tune.apply_tuned(ctx, self.layers, objective=self.tuned_objective)
            table = tune.load_hints(objective=self.tuned_objective)
            self.n_tile_hints = sum(len(table[n]) for n in self.tuned)
        self.descs = (B.LayerDesc * L)(*[B.make_desc(wl) for wl in self.layers])
        self.w_host, self.w_dev, self.g_dev = [], [], []
        w_arr, g_arr = (B.Weights * L)(), (B.WGrads * L)()
        for l, wl in enumerate(self.layers):
            wh = synth.make_weights(wl, seed, l)
            wd = {k: _to_dev(v, wl.dtype) for k, v in wh.items()}
            gd = {k: torch.zeros(v.shape, dtype=torch.float32, device="cuda") for k, v in wh.items()}
            self.w_host.append(wh); self.w_dev.append(wd); self.g_dev.append(gd)
            w_arr[l] = B.Weights(**{k: v.data_ptr() for k, v in wd.items()})
            g_arr[l] = B.WGrads(**{k: v.data_ptr() for k, v in gd.items()})
        self.w_arr, self.g_arr = w_arr, g_arr
        self.stash_mem, stash_arr = [], (B.Stash * (L * n_mb))()
        for l in range(L):
            nbytes = ctx.stash_bytes(self.descs[l])
            for mb in range(n_mb):
                m = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
                self.stash_mem.append(m)
                stash_arr[l * n_mb + mb] = B.Stash(base=m.data_ptr(), bytes=nbytes)
        self.stash_arr = stash_arr
        self.chain_break = list(chain_break) if chain_break is not None else [0] * (L + 1)
        # slot l (l < L) holds the input of layer l, slot L the output of the last layer; a layer that ends a
        # chain in the middle of the stage gets its own output / upstream-gradient ("tail") slots
        self.act, self.grad, self.tail_act, self.tail_grad = [], [], {}, {}
        act_arr, grad_arr = (C.c_void_p * ((L + 1) * n_mb))(), (C.c_void_p * ((L + 1) * n_mb))()
        tail_act_arr, tail_grad_arr = (C.c_void_p * (L * n_mb))(), (C.c_void_p * (L * n_mb))()

        def new_pair(wl):
            td = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
            a = torch.zeros((wl.seq, wl.hidden), dtype=td, device="cuda")
            return a, torch.zeros_like(a)

        for l in range(L + 1):
            wl_shape = self.layers[l] if l < L else self.layers[L - 1]
            for mb in range(n_mb):
                a, g = new_pair(wl_shape)
                self.act.append(a); self.grad.append(g)
                act_arr[l * n_mb + mb] = a.data_ptr()
                grad_arr[l * n_mb + mb] = g.data_ptr()
        for l in range(L - 1):
            if self.chain_break[l + 1]:
                for mb in range(n_mb):
                    a, g = new_pair(self.layers[l])
                    self.tail_act[(l, mb)], self.tail_grad[(l, mb)] = a, g
                    tail_act_arr[l * n_mb + mb] = a.data_ptr()
                    tail_grad_arr[l * n_mb + mb] = g.data_ptr()
        self.act_arr, self.grad_arr = act_arr, grad_arr
        self.tail_act_arr, self.tail_grad_arr = tail_act_arr, tail_grad_arr
        self.cb_arr = (C.c_int32 * (L + 1))(*self.chain_break)
        self.stage = B.Stage(n_layers=L, n_microbatches=n_mb, desc=self.descs, w=w_arr, g=g_arr, stash=stash_arr,
                             act=act_arr, grad=grad_arr, chain_break=self.cb_arr, tail_act=tail_act_arr,
                             tail_grad=tail_grad_arr)
        ctx.ensure_workspace(list(self.descs))

    # ---- slots ----------------------------------------------------------------
    def act_slot(self, l: int, mb: int) -> torch.Tensor:
        return self.act[l * self.n_mb + mb]

    def grad_slot(self, l: int, mb: int) -> torch.Tensor:
        return self.grad[l * self.n_mb + mb]

    def chain_out(self, l: int, mb: int) -> torch.Tensor:
        """Output of layer l when it ends a chain in the middle of the stage."""
        return self.tail_act[(l, mb)]

    def chain_out_grad(self, l: int, mb: int) -> torch.Tensor:
        return self.tail_grad[(l, mb)]

    def field(self, l: int, mb: int, name: str) -> torch.Tensor:
        off, n = self.ctx.stash_field(self.descs[l], name)
        raw = self.stash_mem[l * self.n_mb + mb][off:off + n]
        if name in ("STATS1", "STATS2", "LSE", "DELTA"):
            return raw.view(torch.float32)
        return raw.view(torch.bfloat16 if self.layers[l].dtype == "bf16" else torch.float32)

    def chains(self):
        """[(first_layer, last_layer)] of the independent chains of the stage."""
        L = len(self.layers)
        starts = [l for l in range(L) if l == 0 or self.chain_break[l]]
        return [(a, (starts[i + 1] if i + 1 < len(starts) else L) - 1) for i, a in enumerate(starts)]

    def chain_output(self, last_layer: int, mb: int) -> torch.Tensor:
        L = len(self.layers)
        return self.act_slot(L, mb) if last_layer == L - 1 else self.tail_act[(last_layer, mb)]

    def chain_output_grad(self, last_layer: int, mb: int) -> torch.Tensor:
        L = len(self.layers)
        return self.grad_slot(L, mb) if last_layer == L - 1 else self.tail_grad[(last_layer, mb)]

    def load_inputs(self):
        """Seeded N(0,1) inputs of every chain and upstream gradients of every chain end, per microbatch."""
        for ci, (first, last) in enumerate(self.chains()):
            tag = "" if ci == 0 and len(self.chains()) == 1 else f"c{ci}."
            for mb in range(self.n_mb):
                x = synth.make_activation(self.layers[first], self.seed, f"{tag}x.mb{mb}")
                dy = synth.make_activation(self.layers[last], self.seed, f"{tag}dy.mb{mb}")
                self.act_slot(first, mb).copy_(_to_dev(x, self.layers[first].dtype))
                self.chain_output_grad(last, mb).copy_(_to_dev(dy, self.layers[last].dtype))

    def zero_grads(self):
        for gd in self.g_dev:
            for v in gd.values():
                v.zero_()


class Offloader:
    """Page-locked host buffers and the two copy streams (device -> host, host -> device: the link is full
    duplex) for the activation offload of one stage (Section 4.2, last paragraph; Section 4.3).  Buffers are
    allocated on first use and kept."""

    def __init__(self, stg: StageOnDevice):
        self.stg = stg
        self.copy_stream = torch.cuda.Stream()      # device -> host
        self.reload_stream = torch.cuda.Stream()    # host -> device
        self.host, self.alpha, self.done = {}, {}, {}

    def bytes(self, l: int, which: int, alpha: float) -> int:
        return B.offload_bytes(self.stg.descs[l], which, alpha)

    def offload(self, l: int, mb: int, which: int, alpha: float, s_producer) -> int:
        """Enqueues the device -> host copies behind the work already on s_producer; returns the bytes moved."""
        n = self.bytes(l, which, alpha)
        key = (l, mb, which)
        buf = self.host.get(key)
        if buf is None or buf.numel() < n:
            buf = torch.empty(max(n, 1), dtype=torch.uint8, pin_memory=True)
            self.host[key] = buf
        self.alpha[key] = alpha
        self.stg.ctx.stash_offload(self.stg.descs[l], which, alpha, self.stg.stash_arr[l * self.stg.n_mb + mb], buf,
                                   s_producer, self.copy_stream)
        ev = self.done.get(key)
        if ev is None:
            ev = self.done[key] = torch.cuda.Event()
        ev.record(self.copy_stream)
        return n

    def reload(self, l: int, mb: int, which: int, s_consumer) -> None:
        """Enqueues the host -> device copies behind the offload of the same stash; s_consumer waits for them."""
        key = (l, mb, which)
        self.reload_stream.wait_event(self.done[key])
        self.stg.ctx.stash_reload(self.stg.descs[l], which, self.alpha[key], self.stg.stash_arr[l * self.stg.n_mb + mb],
                                  self.host[key], self.reload_stream, s_consumer)


def plan_offload(steps, n_mb: int, forward_stash: bool = True, w_stash: bool = True, min_gap: int = 1, lead: int = 1):
    """Host-side plan of the offload policy of Section 4.2 / 4.3 for a list of braid steps (each a list of ops).

    The W-stash of a microbatch whose weight gradients are separated (B in one step, W in a later one) leaves
    the device right after its B and returns for its W; the forward stash of a microbatch leaves after the step
    that holds its F (unless its B is in the same step) and returns for the step that holds its B.  Only a
    stash whose consumer is at least `min_gap` steps after its producer is moved: the trip to the host and back
    has to fit into that lifespan, or the consumer waits for it (the paper's T_o < T_F condition).  A reload is
    enqueued `lead` steps ahead of its consumer (never before its offload), so that the copy runs under the steps
    before: `lead` should cover the copy's duration, bytes / link rate, in steps, or the consumer waits for the
    rest; a longer lead keeps the stash on the device for longer.

    Returns (before, after): per step index the lists of ("reload", kind, mb) to enqueue before the step is
    issued and of ("offload" | "reload", kind, mb) to enqueue after it, kind in {"fwd", "w"}."""
    kinds = [{(o.kind, o.microbatch) for o in st} for st in steps]
    n = len(steps)
    before, after = [[] for _ in range(n)], [[] for _ in range(n)]

    def consumer(si, mb, consumer_kinds):
        for sj in range(si + 1, n):
            if any((k, mb) in kinds[sj] for k in consumer_kinds):
                return sj
        return None

    for si in range(n):
        for mb in range(n_mb):
            moves = []
            if forward_stash and (B.OP_F, mb) in kinds[si] and (B.OP_B, mb) not in kinds[si] \
                    and (B.OP_BW, mb) not in kinds[si]:
                moves.append(("fwd", consumer(si, mb, (B.OP_B, B.OP_BW))))
            if w_stash and (B.OP_B, mb) in kinds[si]:
                moves.append(("w", consumer(si, mb, (B.OP_W,))))
            for kind, sj in moves:
                if sj is None or sj - si < max(min_gap, 1):
                    continue
                after[si].append(("offload", kind, mb))
                # `lead` steps ahead of the consumer; right behind the offload if that is earlier than the offload
                after[max(si, sj - max(lead, 1))].append(("reload", kind, mb))
    return before, after


def run_sequence_with_offload(ctx: B.Context, stg: StageOnDevice, steps, streams, off: Offloader, alpha: float,
                              forward_stash: bool = True, w_stash: bool = True, min_gap: int = 1, lead: int = 1) -> int:
    """Issues the braid steps of a stage sequence with the moves plan_offload lists.  Returns the bytes copied
    device -> host (the same number returns)."""
    L = len(stg.layers)
    sF, sB, sW = streams
    before, after = plan_offload(steps, stg.n_mb, forward_stash, w_stash, min_gap, lead)
    moved = 0

    def do(action, kind, mb):
        nonlocal moved
        for l in reversed(range(L)):                    # the backward side starts at the last layer
            if action == "offload" and kind == "fwd":
                moved += off.offload(l, mb, B.OFFLOAD_FWD, alpha, sF)
            elif action == "offload":
                moved += off.offload(l, mb, B.OFFLOAD_W_MLP, alpha, sB)
                moved += off.offload(l, mb, B.OFFLOAD_W_ATTN, alpha, sB)
            elif kind == "fwd":
                off.reload(l, mb, B.OFFLOAD_FWD, sB)
            else:
                off.reload(l, mb, B.OFFLOAD_W_MLP, sW)
                off.reload(l, mb, B.OFFLOAD_W_ATTN, sW)

    for si, step in enumerate(steps):
        for m in before[si]:
            do(*m)
        ctx.braid_step(stg.stage, step, sF, sB, sW)
        for m in after[si]:
            do(*m)
    return moved


# ---- op lists -------------------------------------------------------------------
def _layers(n_layers, layers):
    return list(range(n_layers)) if layers is None else list(layers)


def forward_ops(n_layers: int, mb: int, layers=None) -> List[B.Op]:
    """F units of a microbatch over all layers of the stage, or over the given layers (one model chunk)."""
    return [B.Op(B.OP_F, u, l, mb) for l in _layers(n_layers, layers) for u in (B.PRE_ATTN, B.ATTN, B.PRE_MLP, B.MLP)]


def backward_ops(n_layers: int, mb: int, kind: int = B.OP_BW, layers=None) -> List[B.Op]:
    return [B.Op(kind, u, l, mb) for l in reversed(_layers(n_layers, layers))
            for u in (B.MLP, B.PRE_MLP, B.ATTN, B.PRE_ATTN)]


def weight_ops(n_layers: int, mb: int, layers=None) -> List[B.Op]:
    return [B.Op(B.OP_W, u, l, mb) for l in reversed(_layers(n_layers, layers)) for u in (B.MLP, B.ATTN)]


def braid(f_ops: List[B.Op], b_ops: List[B.Op]) -> List[B.Op]:
    """Interleaves a forward and a backward-side list so that the direction changes at every
    TP boundary (Fig. 3): F.PreAttn F.Attn | B.MLP | F.PreMLP F.MLP | B.PreMLP B.Attn | B.PreAttn ...
    W ops in b_ops ride along with the group they are listed in."""
    def groups(ops, enders):
        out, cur = [], []
        only_w = all(o.kind == B.OP_W for o in ops)
        for o in ops:
            cur.append(o)
            if only_w or (o.unit in enders and o.kind != B.OP_W):
                out.append(cur); cur = []
        if cur:
            out.append(cur)
        return out
    fg = groups(f_ops, (B.ATTN, B.MLP))
    bg = groups(b_ops, (B.MLP, B.ATTN))
    out = []
    for i in range(max(len(fg), len(bg))):
        if i < len(fg):
            out += fg[i]
        if i < len(bg):
            out += bg[i]
    return out


def stage_sequence(n_layers: int, n_mb: int, warmup: int = 1) -> List[List[B.Op]]:
    """One stage's projection of the three-phase schedule (Section 4.2), as a list of braid steps
    exercising every block kind the paper names: warm-up F, F&B with W separated, F&W, steady
    F&BW (W separation off), degraded BW / B, cool-down W.  For 8 microbatches and warmup = 1:
        F0; F1|B0; F2|B1; F3|W0; F4|BW2; F5|BW3; F6|BW4; F7|BW5; BW6; B7; W1; W7
    `warmup` is the number of forward passes in flight before the first backward pass (Appendix A): 1 is the
    memory-efficient warm-up (one extra forward, then overlapped F&B at once), larger values the
    throughput-efficient one (more microbatches in flight, more stashes alive), e.g. warmup = 2:
        F0; F1; F2|B0; F3|B1; F4|W0; F5|BW2; F6|BW3; F7|BW4; BW5; BW6; B7; W1; W7
    Runs too short for the pattern (n_mb < warmup + 3) fall back to F0; F1|BW0; ...; BW(last)."""
    F = lambda i: forward_ops(n_layers, i)
    Bk = lambda j, k: backward_ops(n_layers, j, k)
    W = lambda j: weight_ops(n_layers, j)
    k = max(1, warmup)
    if n_mb < k + 3:
        steps = [F(0)]
        for i in range(1, n_mb):
            steps.append(braid(F(i), Bk(i - 1, B.OP_BW)))
        steps.append(Bk(n_mb - 1, B.OP_BW))
        return steps
    steps = [F(i) for i in range(k)]
    steps += [braid(F(k), Bk(0, B.OP_B)), braid(F(k + 1), Bk(1, B.OP_B)), braid(F(k + 2), W(0))]
    for i in range(k + 3, n_mb):
        steps.append(braid(F(i), Bk(i - k - 1, B.OP_BW)))
    for j in range(n_mb - k - 1, n_mb - 1):
        steps.append(Bk(j, B.OP_BW))
    steps.append(Bk(n_mb - 1, B.OP_B))
    steps.append(W(1))
    steps.append(W(n_mb - 1))
    return steps


def two_chunk_sequence(n_layers: int, first_of_chunk1: int, n_mb: int, pattern: int = 2) -> List[List[B.Op]]:
    """Braid steps of a device that holds two model chunks (layers [0, first_of_chunk1) and the rest; the
    "V" shape of Section 4.1: a microbatch passes chunk 0, later chunk 1, and returns through chunk 1, then
    chunk 0), built after either pattern of Section 4.1:
      pattern 2 (the paper's choice): forward and backward units of the SAME chunk, different microbatches:
          F(c0,0); F(c1,0); F(c0,1); then for i = 1 ..: F(c1,i)|BW(c1,i-1); F(c0,i+1)|BW(c0,i-1)
      pattern 1: forward units of one chunk with backward units of the OTHER:
          ... then for i = 1 ..: F(c0,i+1)|BW(c1,i-1); F(c1,i)|BW(c0,i-1)
    Both issue the same units; only the pairing differs.  When the chunks hold different numbers of units
    (a vision encoder and language-model layers) pattern 1 pairs lists of unequal length."""
    c0, c1 = range(first_of_chunk1), range(first_of_chunk1, n_layers)
    F = lambda c, i: forward_ops(n_layers, i, c)
    BW = lambda c, j: backward_ops(n_layers, j, B.OP_BW, c)
    if n_mb < 2:
        return [F(c0, 0), F(c1, 0), BW(c1, 0), BW(c0, 0)]
    steps = [F(c0, 0), F(c1, 0), F(c0, 1)]
    for i in range(1, n_mb):
        nxt = F(c0, i + 1) if i + 1 < n_mb else []
        if pattern == 2:
            steps.append(braid(F(c1, i), BW(c1, i - 1)))
            steps.append(braid(nxt, BW(c0, i - 1)))
        else:
            steps.append(braid(nxt, BW(c1, i - 1)))
            steps.append(braid(F(c1, i), BW(c0, i - 1)))
    steps += [BW(c1, n_mb - 1), BW(c0, n_mb - 1)]
    return steps


def peak_in_flight(steps: List[List[B.Op]], n_layers: int) -> int:
    """Largest number of (layer, microbatch) stashes alive at once over a list of braid steps: a stash is
    alive from the step that holds the layer's first forward unit to the step that holds its last
    weight-gradient unit (BW counts as both)."""
    first, last = {}, {}
    for si, st in enumerate(steps):
        for o in st:
            key = (o.layer, o.microbatch)
            if o.kind == B.OP_F:
                first.setdefault(key, si)
            if o.kind in (B.OP_W, B.OP_BW) and o.unit == B.ATTN:
                last[key] = si
    peak = 0
    for si in range(len(steps)):
        peak = max(peak, sum(1 for key in first if first[key] <= si <= last.get(key, len(steps))))
    return peak
