"""Host-side checks of the activation offload (no GPU): the byte count the library plans equals the leading
share of exactly those stashed activations that the oracle's deferred units read, and bad arguments are
rejected."""
import ctypes as C

import numpy as np
import pytest

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import binding as B, synth
from oracle import stp_oracle as O
from harness import oracle_cfg

GRANULE = 256


class Recorder(dict):
    """A stash that remembers which entries were read."""

    def __init__(self, *a, **k):
        super().__init__(*a, **k)
        self.reads = set()

    def __getitem__(self, key):
        self.reads.add(key)
        return super().__getitem__(key)


def oracle_reads(wl):
    """Stash keys read by the oracle's W units (per unit) and by its whole backward side."""
    # which entries are read depends on the layer's kind (norm, activation, biases, rope, head grouping),
    # not on its size: take the reads on a small layer of the same kind
    from dataclasses import replace
    group = wl.heads_local // (wl.kv_heads or wl.heads_local)
    wl = replace(wl, hidden=32, heads_local=2 * group, kv_heads=(2 if wl.kv_heads else 0), head_dim=8, ffn_local=48, seq=8)
    cfg = oracle_cfg(wl)
    s = 8
    rng = np.random.default_rng(0)
    W = synth.make_weights(wl, 0, 0)
    W = {k: np.asarray(v, np.float64) for k, v in W.items()}
    X = rng.standard_normal((s, wl.hidden))
    st = {}
    O.forward_unit(cfg, O.PRE_ATTN, W, st, x_in=X)
    xa = O.forward_unit(cfg, O.ATTN, W, st, x_resid=X)
    O.forward_unit(cfg, O.PRE_MLP, W, st, x_in=xa)
    O.forward_unit(cfg, O.MLP, W, st, x_resid=xa)
    fwd_keys = set(st)
    rec = Recorder(st)
    dO = rng.standard_normal((s, wl.hidden))
    dz = O.backward_input_unit(cfg, O.MLP, W, rec, dO)
    dxa = O.backward_input_unit(cfg, O.PRE_MLP, W, rec, dz, d_resid=dO, grads={})
    dxl = O.backward_input_unit(cfg, O.ATTN, W, rec, dxa)
    O.backward_input_unit(cfg, O.PRE_ATTN, W, rec, dxl, d_resid=dxa, grads={})
    b_reads = set(rec.reads)
    w_reads = {}
    for unit in (O.MLP, O.ATTN):
        r = Recorder(dict(rec))
        O.backward_weight_unit(cfg, unit, r, dO if unit == O.MLP else dxa, {})
        w_reads[unit] = set(r.reads)
    return fwd_keys, b_reads, w_reads


# stash entry of the oracle -> bytes of the field that holds it on the device
def field_bytes(wl, key, seq):
    es = 2 if wl.dtype == "bf16" else 4
    T = seq
    qkv_w = (wl.heads_local + 2 * (wl.kv_heads or wl.heads_local)) * wl.head_dim
    return {"x_ln": T * wl.hidden * es, "z_ln": T * wl.hidden * es, "x_attn": T * wl.hidden * es,
            "ctx": T * wl.heads_local * wl.head_dim * es, "qkv": T * qkv_w * es, "dqkv": T * qkv_w * es,
            "h": T * wl.ffn_local * es, "hu": T * wl.ffn_local * es, "g": T * wl.ffn_local * es,
            "dh": T * wl.ffn_local * es, "dhu": T * wl.ffn_local * es,
            "stats": T * 2 * 4, "lse": wl.heads_local * T * 4}[key]


def share(nbytes, alpha):
    want = int(np.ceil(np.float32(alpha).astype(np.float64) * nbytes))
    return min(nbytes, (want + GRANULE - 1) // GRANULE * GRANULE)


WLS = ["tiny", "gpt7b_tp8", "gqa12b_tp4", "llama13b_tp4"]


@pytest.mark.parametrize("name", WLS)
@pytest.mark.parametrize("alpha", [0.0, 0.1, 0.37, 0.5, 1.0])
def test_planned_bytes_are_the_share_of_what_the_deferred_units_read(name, alpha):
    wl = synth.WORKLOADS[name]
    desc = B.make_desc(wl)
    fwd_keys, b_reads, w_reads = oracle_reads(wl)
    # W sets: what the W unit reads from the stash (its dy operand is not a stash entry of the oracle)
    mlp = sorted(w_reads[O.MLP])
    attn = sorted(w_reads[O.ATTN])
    assert set(mlp) <= {"g", "z_ln", "dh", "dhu"} and set(attn) == {"ctx", "x_ln", "dqkv"}
    exp_mlp = sum(share(field_bytes(wl, k, wl.seq), alpha) for k in mlp)
    exp_attn = sum(share(field_bytes(wl, k, wl.seq), alpha) for k in attn)
    assert B.offload_bytes(desc, B.OFFLOAD_W_MLP, alpha) == exp_mlp
    assert B.offload_bytes(desc, B.OFFLOAD_W_ATTN, alpha) == exp_attn
    # forward set: what the forward units wrote and the backward side (B or W) reads; q, k, v share one
    # field; the layer input x is the caller's activation slot, not a stash field; the device also keeps the
    # normalisation statistics and the softmax log-sum-exp, which the oracle recomputes
    used = (b_reads | w_reads[O.MLP] | w_reads[O.ATTN]) & fwd_keys
    keys = sorted({"qkv" if k in ("q", "k", "v") else k for k in used} - {"x"})
    exp_fwd = sum(share(field_bytes(wl, k, wl.seq), alpha) for k in keys)
    exp_fwd += 2 * share(field_bytes(wl, "stats", wl.seq), alpha) + share(field_bytes(wl, "lse", wl.seq), alpha)
    assert B.offload_bytes(desc, B.OFFLOAD_FWD, alpha) == exp_fwd


def test_every_unit_result_of_the_forward_pass_is_in_the_forward_set():
    """x_attn, x_ln, z_ln, q, k, v, ctx, h, g (and hu) are all read again by the backward side."""
    wl = synth.WORKLOADS["llama13b_tp4"]
    fwd_keys, b_reads, w_reads = oracle_reads(wl)
    used = (b_reads | w_reads[O.MLP] | w_reads[O.ATTN]) & fwd_keys
    assert used == {"x", "x_ln", "q", "k", "v", "ctx", "x_attn", "z_ln", "h", "hu", "g"}


@pytest.mark.parametrize("which,alpha", [(7, 0.5), (-1, 0.5), (0, -0.1), (1, 1.5), (2, float("nan"))])
def test_bad_arguments_are_rejected(which, alpha):
    desc = B.make_desc(synth.WORKLOADS["tiny"])
    n = C.c_size_t(123)
    assert B.lib().stp_offload_bytes(C.byref(desc), which, alpha, C.byref(n)) == 1   # STP_EINVAL
    assert B.lib().stp_offload_bytes(C.byref(desc), 0, 0.5, None) == 1


def test_alpha_is_monotone_and_full_at_one():
    wl = synth.WORKLOADS["gpt7b_tp8"]
    desc = B.make_desc(wl)
    prev = 0
    for a in np.linspace(0, 1, 21):
        n = B.offload_bytes(desc, B.OFFLOAD_W_MLP, float(a))
        assert n >= prev
        prev = n
    es = 2
    assert prev == wl.seq * (wl.hidden + 2 * wl.ffn_local) * es


# ---- the offload policy over a stage sequence (host logic) -------------------------------------------------
from paper_2510_27257_amd.stage import plan_offload, stage_sequence


@pytest.mark.parametrize("n_mb", [4, 8, 12])
@pytest.mark.parametrize("min_gap", [1, 2, 3])
@pytest.mark.parametrize("sets", [(True, True), (False, True), (True, False)])
@pytest.mark.parametrize("lead", [1, 3, 100])
def test_offload_plan_pairs_every_move_and_respects_lifespans(n_mb, min_gap, sets, lead):
    steps = stage_sequence(2, n_mb)
    kinds = [{(o.kind, o.microbatch) for o in st} for st in steps]
    before, after = plan_offload(steps, n_mb, forward_stash=sets[0], w_stash=sets[1], min_gap=min_gap, lead=lead)
    assert all(not b for b in before)
    out = {}
    n_moves = 0
    for si in range(len(steps)):
        # a consumer in this step must find its stash on the device
        for mb in range(n_mb):
            if (B.OP_B, mb) in kinds[si] or (B.OP_BW, mb) in kinds[si]:
                assert ("fwd", mb) not in out
            if (B.OP_W, mb) in kinds[si]:
                assert ("w", mb) not in out
        for action, kind, mb in after[si]:
            if action == "offload":
                assert (kind, mb) not in out
                # its producer is in this step, its consumer at least min_gap steps later
                prod = (B.OP_F, mb) if kind == "fwd" else (B.OP_B, mb)
                assert prod in kinds[si]
                cons = (B.OP_B, B.OP_BW) if kind == "fwd" else (B.OP_W,)
                sj = next(j for j in range(si + 1, len(steps)) if any((k, mb) in kinds[j] for k in cons))
                assert sj - si >= min_gap
                out[(kind, mb)] = (si, sj)
                n_moves += 1
            else:
                s_off, sj = out.pop((kind, mb))               # its offload came first (earlier step, or earlier in this list)
                assert si == max(s_off, sj - lead)            # `lead` steps ahead of the consumer, never before the offload
        if not sets[0]:
            assert all(k != "fwd" for _, k, _ in after[si])
        if not sets[1]:
            assert all(k != "w" for _, k, _ in after[si])
    assert not out
    # what must be there: with every lifespan allowed, each separated W and each forward pass moves once
    if min_gap == 1:
        n_w = sum(1 for st in kinds for (k, mb) in st if k == B.OP_B)
        n_f = sum(1 for si, st in enumerate(kinds) for (k, mb) in st
                  if k == B.OP_F and (B.OP_B, mb) not in st and (B.OP_BW, mb) not in st)
        assert n_moves == (n_w if sets[1] else 0) + (n_f if sets[0] else 0)


def test_long_lived_w_stash_of_the_canonical_sequence():
    """8 microbatches: only microbatch 1's weight gradients wait 8 steps (B in step 2, W in step 10)."""
    steps = stage_sequence(4, 8)
    _, after = plan_offload(steps, 8, forward_stash=False, w_stash=True, min_gap=3)
    moves = [(si, m) for si, a in enumerate(after) for m in a]
    assert moves == [(2, ("offload", "w", 1)), (9, ("reload", "w", 1))]
    _, after = plan_offload(steps, 8, forward_stash=False, w_stash=True, min_gap=3, lead=4)
    assert [(si, m) for si, a in enumerate(after) for m in a] == [(2, ("offload", "w", 1)), (6, ("reload", "w", 1))]
