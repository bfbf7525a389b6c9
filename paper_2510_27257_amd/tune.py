"""Measured tile preferences for the bf16 GEMMs of a braided block.

Inside a braided block (Section 3) the GEMMs of the F, B and W units share the GPU with each other and with the
attention and normalisation kernels, and which workgroup tile is fastest for a GEMM there depends on what runs
beside it: a tile that fills the compute units in whole rounds when the GEMM is alone only stretches every tile
when the units are shared, and a big tile that leaves a round half empty costs nothing when other streams fill
it.  The library's own choice is a rule of thumb; this module measures instead: coordinate descent over the
tile of each of a layer's twelve GEMM shapes, the objective being the time of the thing that will run.  Two
objectives, because what is best for one is not best for the other: "block", one layer's F of one microbatch
braided with the full backward of another and issued back to back, so that all three streams stay busy; and
"stage", a pipeline stage's whole sequence of steps (Section 4.2: warm-up F, F&B, F&W, steady F&BW over several
layers, cool-down BW / B / W), where for much of the time only two streams have work.  The result goes to the
context through `stp_gemm_tile_hint` (results do not depend on the tile, only the time does) and can be kept in
a JSON file, one table per objective.

    python -m paper_2510_27257_amd.tune --workloads gqa12b_tp4 gqa26b_tp8 --out paper_2510_27257_amd/tuned_tiles.json
    python -m paper_2510_27257_amd.tune --objective stage --workloads gpt7b_tp8_s4096

needs a GPU; `load_hints` / `apply_hints` do not."""
from __future__ import annotations

import argparse
import json
import os
import time
from typing import Callable, Dict, List, Tuple

from . import binding as B
from . import synth

TILES: List[Tuple[int, int]] = [(256, 256), (128, 256), (256, 128), (128, 128)]
WIDE_TILE = (192, 256)          # only with a k-contiguous A operand (a_trans = 0)
TUNED_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tuned_tiles.json")

Shape = Tuple[int, int, int, int, int]          # M, N, K, a_trans, b_trans


def layer_gemm_shapes(wl: synth.Workload, mbsz: int = 1) -> Dict[str, Shape]:
    """The GEMMs of one layer's F, B and W units as the units call stp_gemm: forward A[T,in] B[in,out]; activation
    gradients with the weight read transposed; weight gradients contracting over the tokens."""
    T, h, a, f, q = wl.seq * mbsz, wl.hidden, wl.attn_local, wl.ffn_local, wl.qkv_local
    return {"qkv_f": (T, q, h, 0, 0), "out_f": (T, h, a, 0, 0), "fc1_f": (T, f, h, 0, 0), "fc2_f": (T, h, f, 0, 0),
            "fc2_b": (T, f, h, 0, 1), "fc1_b": (T, h, f, 0, 1), "out_b": (T, a, h, 0, 1), "qkv_b": (T, h, q, 0, 1),
            "fc2_w": (f, h, T, 1, 0), "fc1_w": (h, f, T, 1, 0), "out_w": (a, h, T, 1, 0), "qkv_w": (h, q, T, 1, 0)}


def apply_hints(ctx: B.Context, hints: Dict[str, str]) -> None:
    """hints: "M,N,K,a_trans,b_trans" -> "TMxTN"."""
    for key, tile in hints.items():
        M, N, K, at, bt = (int(v) for v in key.split(","))
        tm, tn = (int(v) for v in tile.split("x"))
        ctx.gemm_tile_hint(M, N, K, at, bt, tm, tn)


OBJECTIVES = {"block": "workloads", "stage": "stage_workloads"}      # objective -> its table in the file


def load_hints(path: str = TUNED_FILE, objective: str = "block") -> Dict[str, Dict[str, str]]:
    """workload name -> hints measured for this objective; empty if the file is not there."""
    if objective not in OBJECTIVES:
        raise ValueError(f"objective {objective!r}: one of {sorted(OBJECTIVES)}")
    if not os.path.exists(path):
        return {}
    with open(path) as f:
        return json.load(f).get(OBJECTIVES[objective], {})


def apply_tuned(ctx: B.Context, workloads, path: str = TUNED_FILE, objective: str = "block") -> List[str]:
    """Applies the stored hints of every named workload that has an entry for this objective (an empty entry
    says that the library's own choice measured best); returns the names that had one."""
    table, used = load_hints(path, objective), []
    for wl in workloads:
        name = wl if isinstance(wl, str) else wl.name
        if name in table and name not in used:
            apply_hints(ctx, table[name])
            used.append(name)
    return used


def descend(ctx: B.Context, shapes: Dict[str, Shape], run: Callable[[], float], passes: int = 2,
            gain: float = 0.004, log: Callable[[str], None] = lambda s: None) -> Tuple[Dict[str, str], float, float]:
    """Coordinate descent: for each shape in turn, every tile; a tile stays if the block gets faster by more than
    `gain` against a fresh measurement of the best so far (the clocks drift over a run); at the end the whole
    set has to beat the library's own choice by `gain` again, or nothing is kept.  Returns (hints, time with the
    library's own choice, time with the hints)."""
    ctx.gemm_tile_hints_clear()
    base = min(run(), run())
    unique: Dict[Shape, str] = {}
    for name, shape in shapes.items():            # two GEMMs of one shape share their hint
        unique.setdefault(shape, name)
    cur: Dict[Shape, Tuple[int, int]] = {}
    for p in range(passes):
        changed = False
        for shape, name in unique.items():
            M, N, K, at, bt = shape
            best = min(run(), run())
            for tile in TILES + ([WIDE_TILE] if not at else []):
                if cur.get(shape) == tile:
                    continue
                ctx.gemm_tile_hint(M, N, K, at, bt, *tile)
                ms = min(run(), run())
                if ms < best * (1.0 - gain):
                    best, changed = ms, True
                    cur[shape] = tile
                    log(f"  pass {p}: {name} {M}x{N}x{K} -> {tile[0]}x{tile[1]}: {ms:.4f} ms")
                elif shape in cur:
                    ctx.gemm_tile_hint(M, N, K, at, bt, *cur[shape])
                else:
                    ctx.gemm_tile_hint(M, N, K, at, bt, 0, 0)
        if not changed:
            break
    final = min(run(), run())
    hints = {",".join(str(v) for v in shape): f"{t[0]}x{t[1]}" for shape, t in cur.items()}
    if hints:                                     # the whole set against the library's choice once more: single
        ctx.gemm_tile_hints_clear()               # steps of `gain` can be drift, and then the set is dropped
        base = min(run(), run())
        if final > base * (1.0 - gain):
            log(f"  dropped: {final:.4f} ms with {len(hints)} hints against {base:.4f} ms without")
            return {}, base, base
        apply_hints(ctx, hints)
    return hints, base, final


def tune_workload(ctx: B.Context, wl: synth.Workload, steps: int = 150, log=print) -> Tuple[Dict[str, str], float, float]:
    """Tunes the block F(mb 1) | B+W(mb 0) of one layer of this workload on three streams."""
    import torch
    from .stage import StageOnDevice, backward_ops, braid, forward_ops
    stg = StageOnDevice(ctx, [wl], n_mb=2, seed=0, tuned_tiles=False)
    stg.load_inputs()
    streams = [torch.cuda.Stream() for _ in range(3)]
    s0 = torch.cuda.current_stream()
    ctx.braid_reset()
    ctx.braid_step(stg.stage, forward_ops(1, 0), s0, s0, s0)
    torch.cuda.synchronize()
    ops = braid(forward_ops(1, 1), backward_ops(1, 0, B.OP_BW))
    arr = (B.Op * len(ops))(*ops)

    def run() -> float:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            ctx.braid_step(stg.stage, arr, *streams)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    for _ in range(2):
        run()
    return descend(ctx, layer_gemm_shapes(wl), run, log=log)


def tune_stage(ctx: B.Context, models, n_mb: int = 8, reps: int = 0, log=print) -> Tuple[Dict[str, str], float, float]:
    """Tunes the whole sequence of steps of one pipeline stage that holds `models` (one workload per layer; where
    the token or hidden size changes from one layer to the next, the chain of activations is cut there)."""
    import torch
    from .stage import StageOnDevice, stage_sequence
    cut = [0] + [int((a.seq, a.hidden) != (b.seq, b.hidden)) for a, b in zip(models, models[1:])] + [0]
    stg = StageOnDevice(ctx, models, n_mb=n_mb, seed=0, chain_break=cut, tuned_tiles=False)
    stg.load_inputs()
    streams = [torch.cuda.Stream() for _ in range(3)]
    steps = [(B.Op * len(st))(*st) for st in stage_sequence(len(models), n_mb)]

    def run() -> float:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):                     # reps: the enclosing function's, fixed before the descent
            ctx.braid_reset()
            for arr in steps:
                ctx.braid_step(stg.stage, arr, *streams)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    if reps <= 0:                                 # a measurement of a quarter of a second at least
        reps = 4
        run()
        reps = max(4, int(250.0 / run()) + 1)
    for _ in range(2):
        run()
    shapes: Dict[str, Shape] = {}
    for wl in models:
        for name, shape in layer_gemm_shapes(wl).items():
            shapes.setdefault(f"{wl.name}.{name}", shape)
    return descend(ctx, shapes, run, log=log)


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--workloads", nargs="+", required=True,
                    help="block: each is tuned by itself; stage: the layers of ONE stage, each name --layers times")
    ap.add_argument("--objective", choices=sorted(OBJECTIVES), default="block")
    ap.add_argument("--layers", type=int, default=4, help="stage: layers per named workload")
    ap.add_argument("--microbatches", type=int, default=8, help="stage: microbatches of the sequence")
    ap.add_argument("--out", default=TUNED_FILE)
    ap.add_argument("--steps", type=int, default=150)
    args = ap.parse_args()
    import torch
    if not torch.cuda.is_available():
        raise SystemExit("tuning needs a GPU")
    table = {"what": "tile preferences of the bf16 GEMMs beside other streams, measured by "
                     "`python -m paper_2510_27257_amd.tune`; key: M,N,K,a_trans,b_trans; `workloads`: for one "
                     "layer's braided block issued back to back; `stage_workloads`: for a stage's whole "
                     "sequence of steps (an empty entry: the library's own choice measured best)",
             "workloads": load_hints(args.out, "block"), "stage_workloads": load_hints(args.out, "stage"),
             "block_ms": {}, "stage_ms": {}}
    if os.path.exists(args.out):
        with open(args.out) as f:
            old = json.load(f)
            table["block_ms"] = old.get("block_ms", {})
            table["stage_ms"] = old.get("stage_ms", {})
    ctx = B.Context(0)
    if args.objective == "stage":
        wls = [synth.WORKLOADS[n] for n in args.workloads]
        models = [wl for wl in wls for _ in range(args.layers)]
        tag = "+".join(args.workloads)
        print(f"[stage {tag}]", flush=True)
        hints, base, final = tune_stage(ctx, models, args.microbatches, log=lambda s: print(s, flush=True))
        print(f"[stage {tag}] library's choice {base:.4f} ms, tuned {final:.4f} ms, {len(hints)} hints", flush=True)
        for wl in wls:                       # each workload keeps the hints of its own shapes
            own = {",".join(str(v) for v in sh) for sh in layer_gemm_shapes(wl).values()}
            table["stage_workloads"][wl.name] = {k: v for k, v in hints.items() if k in own}
        table["stage_ms"][tag] = {"library_choice": round(base, 4), "tuned": round(final, 4)}
        args.workloads = []
    for name in args.workloads:
        wl = synth.WORKLOADS[name]
        print(f"[{name}]", flush=True)
        hints, base, final = tune_workload(ctx, wl, args.steps, log=lambda s: print(s, flush=True))
        print(f"[{name}] library's choice {base:.4f} ms, tuned {final:.4f} ms, {len(hints)} hints", flush=True)
        table["workloads"][name] = hints
        table["block_ms"][name] = {"library_choice": round(base, 4), "tuned": round(final, 4)}
        ctx.gemm_tile_hints_clear()
        torch.cuda.empty_cache()
    ctx.close()
    os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
    with open(args.out, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    print("wrote", args.out)


if __name__ == "__main__":
    main()
