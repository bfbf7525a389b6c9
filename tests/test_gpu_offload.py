"""Activation offload and reload on the GPU: the bytes come back exactly, the device copy is not needed in
between (it is overwritten), and a stage sequence with offloaded W-stashes and forward stashes produces the
same bits as the sequence without."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import binding as B, synth
from paper_2510_27257_amd.stage import Offloader, StageOnDevice, run_sequence_with_offload, stage_sequence
from paper_2510_27257_amd.synth import Workload
from harness import TOL, oracle_cfg, oracle_layer_pass, rel_err, to_host

GRANULE = 256
W_ATTN_FIELDS = ["X_LN", "CTX", "DQKV"]
FWD_FIELDS = ["X_LN", "STATS1", "QKV", "CTX", "LSE", "Z_LN", "STATS2", "H", "HU", "G", "X_ATTN"]


def w_mlp_fields(wl):
    return ["Z_LN", "G", "DH"] + (["DHU"] if wl.act == "swiglu" else [])


def moved_ranges(ctx, desc, fields, alpha):
    """(offset, bytes) of the leading share of every field, by the rule the header states."""
    out = []
    for f in fields:
        off, n = ctx.stash_field(desc, f)
        want = int(np.ceil(np.float64(np.float32(alpha)) * n))
        take = min(n, (want + GRANULE - 1) // GRANULE * GRANULE)
        if take:
            out.append((off, take))
    return out


@pytest.fixture(scope="module")
def ctx():
    c = stp.Context(0)
    yield c
    torch.cuda.synchronize()
    c.close()


GPT = Workload("g", 512, 2, 128, 1024, 264, 8)
LLAMA = Workload("l", 384, 6, 64, 520, 136, 4, norm="rms", act="swiglu", rope=True, has_bias=False, kv_heads=2)


def fields_of(wl, which):
    if which == B.OFFLOAD_W_ATTN:
        return W_ATTN_FIELDS
    if which == B.OFFLOAD_W_MLP:
        return w_mlp_fields(wl)
    return [f for f in FWD_FIELDS if f != "HU" or wl.act == "swiglu"]


@pytest.mark.parametrize("wl", [GPT, LLAMA], ids=["gpt", "llama_gqa"])
@pytest.mark.parametrize("which", [B.OFFLOAD_W_ATTN, B.OFFLOAD_W_MLP, B.OFFLOAD_FWD])
@pytest.mark.parametrize("alpha", [0.3, 1.0])
def test_round_trip_is_exact_and_does_not_need_the_device_copy(ctx, wl, which, alpha):
    stg = StageOnDevice(ctx, [wl], 1, seed=5)
    stg.load_inputs()
    s0 = torch.cuda.current_stream()
    ctx.braid_reset()
    for step in stage_sequence(1, 1):          # F0 ; BW0 fills every field
        ctx.braid_step(stg.stage, step, s0, s0, s0)
    torch.cuda.synchronize()
    before = stg.stash_mem[0].clone()
    off = Offloader(stg)
    n = off.offload(0, 0, which, alpha, s0)
    ranges = moved_ranges(ctx, stg.descs[0], fields_of(wl, which), alpha)
    assert n == sum(r[1] for r in ranges) == B.offload_bytes(stg.descs[0], which, alpha)
    off.copy_stream.synchronize()
    # host holds the leading shares back to back
    host = off.host[(0, 0, which)]
    exp = torch.cat([before[o:o + b] for o, b in ranges]).cpu()
    assert torch.equal(host[:n], exp)
    # the moved device ranges are dead now: overwrite them, and nothing else
    for o, b in ranges:
        stg.stash_mem[0][o:o + b].fill_(0xA5)
    untouched = stg.stash_mem[0].clone()
    for o, b in ranges:
        untouched[o:o + b] = before[o:o + b]
    assert torch.equal(untouched, before)
    s1 = torch.cuda.Stream()
    off.reload(0, 0, which, s1)
    with torch.cuda.stream(s1):
        after = stg.stash_mem[0].clone()       # ordered behind the reload by the consumer stream's wait
    torch.cuda.synchronize()
    assert torch.equal(after, before)


def run_sequence(ctx, stg, streams, offload=None, alpha=1.0, poison=True):
    """The stage sequence; with `offload` the W-stash of every microbatch whose W is deferred leaves the device
    right after its B and returns right before its W, and every forward stash leaves after its F step and
    returns before the step that holds its B."""
    L, n_mb = len(stg.layers), stg.n_mb
    sF, sB, sW = streams
    ctx.braid_reset()
    stg.zero_grads()
    steps = stage_sequence(L, n_mb)
    kinds = [{(o.kind, o.microbatch) for o in st} for st in steps]
    out_w, out_f = set(), set()
    for si, step in enumerate(steps):
        if offload is not None:
            for mb in range(n_mb):
                b_here = (B.OP_B, mb) in kinds[si] or (B.OP_BW, mb) in kinds[si]
                w_here = (B.OP_W, mb) in kinds[si]
                if mb in out_f and b_here:
                    for l in range(L):
                        offload.reload(l, mb, B.OFFLOAD_FWD, sB)
                    out_f.discard(mb)
                if mb in out_w and w_here:
                    for l in range(L):
                        offload.reload(l, mb, B.OFFLOAD_W_ATTN, sW)
                        offload.reload(l, mb, B.OFFLOAD_W_MLP, sW)
                    out_w.discard(mb)
        ctx.braid_step(stg.stage, step, sF, sB, sW)
        if offload is not None:
            for mb in range(n_mb):
                if (B.OP_F, mb) in kinds[si] and (B.OP_B, mb) not in kinds[si] and (B.OP_BW, mb) not in kinds[si]:
                    for l in range(L):
                        offload.offload(l, mb, B.OFFLOAD_FWD, alpha, sF)
                    out_f.add(mb)
                if (B.OP_B, mb) in kinds[si]:            # B without W: its W comes in a later step
                    for l in range(L):
                        offload.offload(l, mb, B.OFFLOAD_W_ATTN, alpha, sB)
                        offload.offload(l, mb, B.OFFLOAD_W_MLP, alpha, sB)
                    out_w.add(mb)
            if poison:
                # overwrite what has left the device once the copies are through
                offload.copy_stream.synchronize()
                for mb in out_f | out_w:
                    for l in range(L):
                        sets = ([B.OFFLOAD_FWD] if mb in out_f else []) + ([B.OFFLOAD_W_ATTN, B.OFFLOAD_W_MLP] if mb in out_w else [])
                        for which in sets:
                            for o, b in moved_ranges(ctx, stg.descs[l], fields_of(stg.layers[l], which), alpha):
                                stg.stash_mem[l * n_mb + mb][o:o + b].fill_(0xFF)
                torch.cuda.synchronize()
    assert not out_w and not out_f
    torch.cuda.synchronize()


def results(stg):
    out = [t.clone() for t in stg.grad]
    for gd in stg.g_dev:
        out += [gd[k].clone() for k in sorted(gd)]
    return out


@pytest.mark.parametrize("layers,n_mb", [([GPT] * 2, 5), ([LLAMA], 6)], ids=["gpt_x2", "llama_gqa_x1"])
@pytest.mark.parametrize("alpha", [0.4, 1.0])
def test_sequence_with_offload_equals_sequence_without(ctx, layers, n_mb, alpha):
    stg = StageOnDevice(ctx, layers, n_mb, seed=3)
    stg.load_inputs()
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    run_sequence(ctx, stg, streams)
    ref = results(stg)
    off = Offloader(stg)
    run_sequence(ctx, stg, streams, offload=off, alpha=alpha, poison=True)
    got = results(stg)
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
    # and without host synchronisation in between: ordering by the events alone
    run_sequence(ctx, stg, streams, offload=off, alpha=alpha, poison=False)
    got = results(stg)
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
    # the library's own policy runner (reloads enqueued one step ahead, two copy streams)
    ctx.braid_reset()
    stg.zero_grads()
    moved = run_sequence_with_offload(ctx, stg, stage_sequence(len(layers), n_mb), streams, off, alpha)
    torch.cuda.synchronize()
    assert moved > 0
    for a, b in zip(results(stg), ref):
        assert torch.equal(a, b)


def test_weight_gradients_after_reload_match_the_oracle(ctx):
    wl = GPT
    stg = StageOnDevice(ctx, [wl], 4, seed=7)
    stg.load_inputs()
    streams = (torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream())
    off = Offloader(stg)
    run_sequence(ctx, stg, streams, offload=off, alpha=1.0, poison=True)
    cfg = oracle_cfg(wl)
    W = {k: v.astype(np.float64) for k, v in stg.w_host[0].items()}
    grads = {}
    for mb in range(stg.n_mb):
        X = synth.make_activation(wl, 7, f"x.mb{mb}").astype(np.float64)
        dO = synth.make_activation(wl, 7, f"dy.mb{mb}").astype(np.float64)
        oracle_layer_pass(cfg, W, X, dO, grads)
    for k in ("w_fc1", "w_fc2", "w_qkv", "w_o", "b_fc1", "b_qkv"):
        assert rel_err(to_host(stg.g_dev[0][k]), grads[k]) < TOL[wl.dtype], k


def test_errors(ctx):
    stg = StageOnDevice(ctx, [synth.WORKLOADS["tiny"]], 1, seed=1)
    s0 = torch.cuda.current_stream()
    desc, stash = stg.descs[0], stg.stash_arr[0]
    small = torch.empty(16, dtype=torch.uint8, pin_memory=True)
    with pytest.raises(stp.StpError) as e:
        ctx.stash_offload(desc, B.OFFLOAD_W_MLP, 1.0, stash, small, s0, s0)
    assert e.value.status == 1 and "too small" in str(e.value)
    big = torch.empty(1 << 20, dtype=torch.uint8, pin_memory=True)
    for which, alpha in [(9, 0.5), (0, 2.0), (1, -1.0)]:
        with pytest.raises(stp.StpError) as e:
            ctx.stash_reload(desc, which, alpha, stash, big, s0, s0)
        assert e.value.status == 1
    short = B.Stash(base=stash.base, bytes=64)
    with pytest.raises(stp.StpError):
        ctx.stash_offload(desc, B.OFFLOAD_FWD, 0.5, short, big, s0, s0)
    torch.cuda.synchronize()
