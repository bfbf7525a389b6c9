"""Host-side generator and simulator of the synergistic tensor / pipeline schedule (Section 4: "V" flow over two
model chunks per device, warm-up / steady / cool-down phases, braided blocks after pattern (2), weight-gradient
separation in the warm-up and in the degraded phase), and the bridge from a device's program to the braid steps
`stp_braid_step` executes.  No GPU, no torch: plain Python.

Device d of p holds virtual stages d (chunk 0) and 2p-1-d (chunk 1); a microbatch runs forward through virtual
stages 0 .. 2p-1 and backward through 2p-1 .. 0.  A device's program is a list of blocks; a block has at most one
forward part F(chunk, mb), at most one activation-gradient part B(chunk, mb) and any number of weight-gradient
parts W(chunk, mb) (a B with its own W in the same block is the full backward BW).

The program of device d (the figures of the schedule are not in the text; this is the construction the text of
Section 4.2 and Table 1 pin down, derived from the steady-state timetable of the "V" flow in which a device
alternates chunk-1 and chunk-0 blocks):
  warm-up 1   2p+1 plain forward passes, the maximum before the first backward pass can arrive: chunk-1 forward i
              at position 2p-1-2d+2i (i = 0 .. d), chunk-0 forwards elsewhere.  These are the only forward passes
              whose all-reduce is exposed: (2p+1) T_AR, Table 1's TP bubble.
  warm-up 2   until the first chunk-0 backward arrives (p-d-1 rounds; none on the last device): F&B of chunk 1
              with W separated, so that the gradient moves on at once, then F of chunk 0 & the separated W.
              In-flight activations reach 3p-d: Table 1's peak of 3p on device 0.
  steady      F&BW of chunk 1, F&BW of chunk 0, W separation off, while chunk-0 forwards remain.  Optionally the
              last `steady_w_tail` braids of the phase separate and store their W as well (Section 4.2 allows
              separation in the steady phase at the price of the stash it keeps alive until the final steps, which
              is what the offload is for): more stored W to fill the waits of the cool-down phase.
  degraded    chunk-0 forwards exhausted: full backward of chunk 0, F&B of chunk 1 with W separated and stored.
  cool-down   the remaining backward passes as full backward passes (their own W hides the all-reduce); the W
              blocks stored in the degraded phase float into waits that are long enough for them.
It needs m >= 3p microbatches (the paper assumes p << m).

For the simulator only, the two comparison rows of Table 1: `program_1f1b_interleaved` (parallel flow, unsplit
backward; reproduces the table's PP and TP bubbles exactly) and `greedy_zero_bubble_v` (a list-scheduled
Zero-Bubble-V style program; reproduces the table's TP bubble and peak memory).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

Part = Tuple[int, int]          # (chunk, microbatch)


@dataclass
class Block:
    f: Optional[Part] = None
    b: Optional[Part] = None
    w: Tuple[Part, ...] = ()
    start: float = 0.0
    end: float = 0.0

    def name(self) -> str:
        s = []
        if self.f:
            s.append("F%d.%d" % self.f)
        if self.b:
            s.append(("BW" if self.b in self.w else "B") + "%d.%d" % self.b)
        s += ["W%d.%d" % x for x in self.w if x != self.b]
        return "&".join(s)


@dataclass(frozen=True)
class Times:
    """Per model chunk (Section 4.3): forward, activation-gradient, weight-gradient time, and the TP all-reduce
    time of one chunk in one direction."""
    TF: float = 1.0
    TB: float = 1.0
    TW: float = 1.0
    TAR: float = 0.0


def vstage(p: int, d: int, chunk: int, flow: str = "v") -> int:
    """Virtual stage of model chunk `chunk` of device d: the "V" flow folds the second half back (device 0 holds the
    first and the last stage), the parallel flow of interleaved 1F1B runs both halves in device order."""
    if chunk == 0:
        return d
    return 2 * p - 1 - d if flow == "v" else p + d


def device_program(p: int, m: int, d: int, steady_w_tail: int = 0) -> List[Block]:
    """The block list of device d for p devices and m microbatches (see the module docstring)."""
    if p < 1 or not 0 <= d < p:
        raise ValueError("need 0 <= d < p")
    if m < 3 * p:
        raise ValueError("the schedule keeps up to 3p microbatches in flight: need m >= 3p")
    prog: List[Block] = []
    f, b, stored = [0, 0], [0, 0], []

    def F(c):
        i = f[c]
        f[c] += 1
        return (c, i)

    def Bk(c):
        j = b[c]
        b[c] += 1
        return (c, j)

    c1_pos = {2 * p - 1 - 2 * d + 2 * i for i in range(d + 1)}
    for q in range(2 * p + 1):
        prog.append(Block(f=F(1 if q in c1_pos else 0)))
    c, w2_left = 1, p - d - 1
    while b[0] < m or b[1] < m:
        have_f, have_b = f[c] < m, b[c] < m
        steady = f[0] < m
        if c == 0 and w2_left > 0 and have_f:
            w = (stored.pop(0),) if stored else ()
            prog.append(Block(f=F(0), w=w))
            w2_left -= 1
        elif have_f and have_b and f[c] > b[c]:
            left = 2 * (m - f[0]) - (1 if c == 0 else 0)     # steady braids still to come, this one included
            separate = (c == 1 and w2_left > 0) or not steady or left <= steady_w_tail
            bb = Bk(c)
            prog.append(Block(f=F(c), b=bb, w=() if separate else (bb,)))
            if separate:
                stored.append(bb)
        elif have_b and (c == 1 or b[0] < b[1]):      # "V" order: chunk 0 of a microbatch after its chunk 1
            bb = Bk(c)
            prog.append(Block(b=bb, w=(bb,)))
        elif have_f:
            w = (stored.pop(0),) if stored else ()
            prog.append(Block(f=F(c), w=w))
        c = 1 - c
    prog += [Block(w=(x,)) for x in stored]
    return prog


def build(p: int, m: int, steady_w_tail: int = 0) -> List[List[Block]]:
    return [device_program(p, m, d, steady_w_tail) for d in range(p)]


def block_time(blk: Block, t: Times) -> Tuple[float, float]:
    """(duration, exposed all-reduce time inside it).  A braided F&B hides both all-reduces; a W part hides the
    all-reduce of the F or B it shares the block with; a plain F or plain B exposes one."""
    dur = (t.TF if blk.f else 0.0) + (t.TB if blk.b else 0.0) + len(blk.w) * t.TW
    exposed = 0.0
    if (blk.f is None) != (blk.b is None) and not blk.w:
        exposed = t.TAR
    return dur + exposed, exposed


def simulate(p: int, programs: List[List[Block]], t: Times, float_w: bool = True, flow: str = "v",
             atomic_bw: bool = False) -> float:
    """Fills start / end of every block and returns the makespan.  A device runs its blocks in order; F(v, i) waits
    for F(v-1, i), B(v, j) for F(v, j) and B(v+1, j), a W part for its B.  Results leave a block as soon as they
    exist: after T_F (+ exposed all-reduce) for a forward-only block, after T_B for a backward-only block (its W
    parts run last), after T_F + T_B for a braided block (its units interleave).  With float_w a W-only block
    whose B is done moves forward into a wait of at least T_W (the stored weight gradients fill the bubbles of
    the cool-down phase); the programs are reordered in place accordingly.  `flow` names the stage order ("v" or
    "parallel"); with atomic_bw a full backward pass hands its gradient on only when its W part is done too
    (interleaved 1F1B does not split the backward pass)."""
    V = 2 * p

    def vs(p_, d_, c_):          # virtual stage under the flow of this run
        return vstage(p_, d_, c_, flow)

    f_out: Dict[Part, float] = {}
    b_out: Dict[Part, float] = {}
    idx, now = [0] * p, [0.0] * p
    total, done = sum(len(x) for x in programs), 0
    while done < total:
        progress = False
        for d in range(p):
            while idx[d] < len(programs[d]):
                blk = programs[d][idx[d]]
                ready, ok = now[d], True
                if blk.f:
                    v = vs(p, d, blk.f[0])
                    if v > 0:
                        if (v - 1, blk.f[1]) not in f_out:
                            ok = False
                        else:
                            ready = max(ready, f_out[(v - 1, blk.f[1])])
                if ok and blk.b:
                    v = vs(p, d, blk.b[0])
                    if (v, blk.b[1]) not in f_out:
                        ok = False
                    else:
                        ready = max(ready, f_out[(v, blk.b[1])])
                    if ok and v < V - 1:
                        if (v + 1, blk.b[1]) not in b_out:
                            ok = False
                        else:
                            ready = max(ready, b_out[(v + 1, blk.b[1])])
                if ok:
                    for x in blk.w:
                        if x != blk.b:
                            if (vs(p, d, x[0]), x[1]) not in b_out:
                                ok = False
                            else:
                                ready = max(ready, b_out[(vs(p, d, x[0]), x[1])])
                if not ok:
                    break
                w_only = bool(blk.w) and not blk.f and not blk.b
                if float_w and not w_only and ready - now[d] >= t.TW - 1e-9:
                    k = next((k for k in range(idx[d] + 1, len(programs[d]))
                              if programs[d][k].w and not programs[d][k].f and not programs[d][k].b
                              and all(b_out.get((vs(p, d, x[0]), x[1]), float("inf")) <= now[d] + 1e-9
                                      for x in programs[d][k].w)), None)
                    if k is not None:
                        programs[d].insert(idx[d], programs[d].pop(k))
                        continue
                dur, exposed = block_time(blk, t)
                blk.start, blk.end = ready, ready + dur
                now[d] = blk.end
                if blk.f and blk.b:
                    out = ready + t.TF + t.TB
                elif blk.f:
                    out = ready + t.TF + exposed
                else:
                    out = ready + t.TB + exposed + (t.TW if atomic_bw and blk.b in blk.w else 0.0)
                if blk.f:
                    f_out[(vs(p, d, blk.f[0]), blk.f[1])] = out
                if blk.b:
                    b_out[(vs(p, d, blk.b[0]), blk.b[1])] = out
                idx[d] += 1
                done += 1
                progress = True
        if not progress:
            raise RuntimeError("the programs deadlock: " + ", ".join(
                "device %d at %s" % (d, programs[d][idx[d]].name()) for d in range(p) if idx[d] < len(programs[d])))
    return max(now)


def metrics(p: int, programs: List[List[Block]], t: Times) -> List[dict]:
    """Per device, from simulated programs: PP bubble (makespan minus the time its blocks take), TP bubble
    (all-reduce time not hidden inside a block), idle time before its first block, and the peak number of
    chunk-activations held: `peak_activation` counts a (chunk, microbatch) from the end of its forward block to
    the end of the block with its B (what Table 1 calls activation memory, in units of M_a), `peak_with_w_stash`
    until the end of the block with its W (a separated W keeps part of it alive; the paper offloads that part)."""
    T = max(b.end for pr in programs for b in pr)
    out = []
    for d in range(p):
        busy = sum(block_time(b, t)[0] for b in programs[d])
        exposed = sum(block_time(b, t)[1] for b in programs[d])

        def peak(until_w: bool) -> int:
            ev = []
            for blk in programs[d]:
                if blk.f:
                    ev.append((blk.end, 1))
                for x in (blk.w if until_w else ((blk.b,) if blk.b else ())):
                    ev.append((blk.end, -1))
            ev.sort()
            cur = best = 0
            for _, delta in ev:
                cur += delta
                best = max(best, cur)
            return best

        out.append({"pp_bubble": T - busy, "tp_bubble": exposed, "start_idle": programs[d][0].start,
                    "peak_activation": peak(False), "peak_with_w_stash": peak(True)})
    return out


def table1(p: int, t: Times, row: str = "ours", m: int = 0) -> dict:
    """Table 1's closed forms (the paper calls the bubble sizes approximate).  Rows: "ours" (the proposed schedule),
    "1f1b-i" (interleaved 1F1B, two virtual stages) and "zb-v" (Zero Bubble V); the TP bubbles of the latter two
    grow with the number of microbatches m."""
    if row == "ours":
        return {"pp_bubble": (p - 1) * (t.TF + t.TAR + t.TB - t.TW), "tp_bubble": (2 * p + 1) * t.TAR,
                "peak_activation": 3 * p}
    if row == "1f1b-i":
        return {"pp_bubble": (p - 1) * (t.TF + t.TAR + t.TB + t.TW), "tp_bubble": 2 * m * t.TAR,
                "peak_activation": 3 * p - 2}
    if row == "zb-v":
        return {"pp_bubble": (p - 1) * (t.TF + 2 * t.TAR + t.TB - 2 * t.TW), "tp_bubble": 4 * m * t.TAR,
                "peak_activation": 2 * p}
    raise ValueError(row)


# ---- the two comparison rows of Table 1, for the simulator only (nothing of them runs on the GPU) -----------------
def program_1f1b_interleaved(p: int, m: int, d: int) -> List[Block]:
    """Interleaved 1F1B with two virtual stages per device in the parallel flow (device d holds stages d and p + d):
    microbatches go through in groups of p, chunk 0 of a group then its chunk 1; device d runs 2(p-d-1) + p
    forward passes ahead, then alternates one forward and one full backward pass, then drains.  Every forward
    pass is a plain block (its all-reduce is exposed), every backward pass carries its own W (which hides its
    all-reduce): Table 1's 2 m T_AR.  Needs m to be a multiple of p."""
    if m % p:
        raise ValueError("interleaved 1F1B takes the microbatches in groups of p: m must be a multiple of p")

    def slot(k: int, backward: bool) -> Part:
        c = (k // p) % 2
        return (1 - c if backward else c, (k // (2 * p)) * p + k % p)

    total = 2 * m
    warm = min(2 * (p - d - 1) + p, total)
    prog = [Block(f=slot(k, False)) for k in range(warm)]
    for i in range(total - warm):
        prog.append(Block(f=slot(warm + i, False)))
        b = slot(i, True)
        prog.append(Block(b=b, w=(b,)))
    for i in range(total - warm, total):
        b = slot(i, True)
        prog.append(Block(b=b, w=(b,)))
    return prog


def greedy_zero_bubble_v(p: int, m: int, t: Times, cap: Optional[int] = None) -> List[List[Block]]:
    """A Zero-Bubble-V style schedule for the simulator: the "V" flow, forward, activation-gradient and weight-
    gradient passes all separate (every F and every B is a plain block with an exposed all-reduce: Table 1's
    4 m T_AR), at most `cap` chunk-activations alive per device (default 2p, Table 1's peak).  Built by list
    scheduling in simulated time: a free device takes a ready B (the one that became ready first), else a ready F
    if its memory allows (one slot is kept for chunk 1), else a W whose B is done, else waits for the next result; the weight-gradient passes
    so fill the waits.  Returns the programs with their start and end times filled."""
    cap = 2 * p if cap is None else cap
    V = 2 * p
    INF = float("inf")
    f_out: Dict[Part, float] = {}
    b_out: Dict[Part, float] = {}
    progs: List[List[Block]] = [[] for _ in range(p)]
    now = [0.0] * p
    nf, nb = [[0, 0] for _ in range(p)], [[0, 0] for _ in range(p)]
    w_pending: List[List[Part]] = [[] for _ in range(p)]
    alive = [0] * p
    todo = 3 * 2 * m * p
    def candidates(d: int):
        cands = []
        for c in (1, 0):
            j = nb[d][c]
            if j < m:
                v = vstage(p, d, c)
                r = max(f_out.get((v, j), INF), b_out.get((v + 1, j), INF) if v < V - 1 else 0.0)
                if r < INF:
                    cands.append((max(r, now[d]), 0, r, "b", c, j))
        for c in (0, 1):
            i = nf[d][c]
            # one slot stays free for chunk 1, whose forward pass is what lets a backward pass (and with it the
            # release of memory) begin: without it the chunk-0 forwards fill the memory and nothing can move
            if i < m and alive[d] < (cap if c == 1 else cap - 1):
                v = vstage(p, d, c)
                r = f_out.get((v - 1, i), INF) if v > 0 else 0.0
                if r < INF:
                    cands.append((max(r, now[d]), 1, r, "f", c, i))
        if w_pending[d]:
            cands.append((now[d], 2, now[d], "w", *w_pending[d][0]))
        return cands

    while todo:
        # the device that is free first and has something it can start moves next (ties: lowest index)
        d, cands = -1, []
        for x in sorted(range(p), key=lambda x: (now[x], x)):
            cands = candidates(x)
            if cands:
                d = x
                break
        if d < 0:
            raise RuntimeError("the greedy schedule deadlocks (memory cap too small?)")
        # start as early as possible; among those, B before F before W
        start, _, _, kind, c, i = min(cands)
        if kind != "w" and start > now[d] + 1e-12 and w_pending[d] and start - now[d] >= t.TW - 1e-12:
            kind, (c, i), start = "w", w_pending[d][0], now[d]
        if kind == "f":
            blk = Block(f=(c, i), start=start, end=start + t.TF + t.TAR)
            f_out[(vstage(p, d, c), i)] = blk.end
            nf[d][c] += 1
            alive[d] += 1
        elif kind == "b":
            blk = Block(b=(c, i), start=start, end=start + t.TB + t.TAR)
            b_out[(vstage(p, d, c), i)] = blk.end
            nb[d][c] += 1
            alive[d] -= 1
            w_pending[d].append((c, i))
        else:
            blk = Block(w=((c, i),), start=start, end=start + t.TW)
            w_pending[d].pop(0)
        progs[d].append(blk)
        now[d] = blk.end
        todo -= 1
    return progs


def braid_steps(program: Sequence[Block], n_layers: int, first_of_chunk1: int):
    """The op lists `stp_braid_step` takes, one per block, for a stage whose layers [0, first_of_chunk1) are chunk 0
    and the rest chunk 1 (a chain break between them)."""
    from . import binding as B
    from .stage import backward_ops, braid, forward_ops, weight_ops
    chunks = (range(first_of_chunk1), range(first_of_chunk1, n_layers))
    steps = []
    for blk in program:
        f_ops = forward_ops(n_layers, blk.f[1], chunks[blk.f[0]]) if blk.f else []
        b_ops = []
        if blk.b:
            own = blk.b in blk.w
            b_ops += backward_ops(n_layers, blk.b[1], B.OP_BW if own else B.OP_B, chunks[blk.b[0]])
        for x in blk.w:
            if x != blk.b:
                b_ops += weight_ops(n_layers, x[1], chunks[x[0]])
        steps.append(braid(f_ops, b_ops) if f_ops and b_ops else f_ops + b_ops)
    return steps
