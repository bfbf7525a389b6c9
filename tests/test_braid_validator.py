"""Host-only checks: the library loads, exports every declared symbol, and the braid's
sequence validator enforces the ordering rules (Appendix A: the forward microbatch index must
exceed the backward one; units in dependence order; W only for Attn / MLP)."""
import ctypes as C
import os
import re

import pytest

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import synth
from paper_2510_27257_amd.binding import Op, OP_F, OP_B, OP_W, OP_BW, PRE_ATTN, ATTN, PRE_MLP, MLP

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    L = stp.lib()
    header = open(os.path.join(ROOT, "include", "stp.h")).read()
    declared = set(re.findall(r"\b(stp_[a-z_]+)\s*\(", header))
    declared -= {"stp_boundary_fn"}
    assert declared == set(stp.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(L, name) is not None


def test_struct_sizes_match_header():
    assert C.sizeof(stp.LayerDesc) == 16 * 4
    assert C.sizeof(stp.Weights) == 13 * 8 and C.sizeof(stp.WGrads) == 13 * 8
    assert C.sizeof(stp.Op) == 16 and C.sizeof(stp.Stash) == 16
    assert C.sizeof(stp.Stage) == 8 + 9 * 8


def test_desc_checks_and_sizes_need_no_gpu():
    L = stp.lib()
    d = stp.make_desc(synth.WORKLOADS["gpt7b_tp8"])
    assert L.stp_check_desc(C.byref(d)) == 0
    n = C.c_size_t()
    assert L.stp_stash_bytes(C.byref(d), C.byref(n)) == 0
    T, h, a, f = 6144, 4096, 512, 2048
    lower = 2 * T * (6 * h + 2 * 3 * a + 2 * a + 3 * f)
    assert lower <= n.value < lower * 1.02
    offs = []
    for i, name in enumerate(stp.STASH_FIELDS):
        off, sz = C.c_size_t(), C.c_size_t()
        assert L.stp_stash_field(C.byref(d), i, C.byref(off), C.byref(sz)) == 0
        assert off.value % 256 == 0
        offs.append((off.value, sz.value))
    for (o1, s1), (o2, _) in zip(offs, offs[1:]):
        assert o1 + s1 <= o2
    assert offs[-1][0] + offs[-1][1] <= n.value
    for field, val, status in [("hidden", 4100, 2), ("head_dim", 96, 2), ("seq", 6143, 2), ("dtype", 5, 1),
                               ("tp", 0, 2), ("norm", 3, 1)]:
        bad = stp.make_desc(synth.WORKLOADS["gpt7b_tp8"])
        setattr(bad, field, val)
        assert L.stp_check_desc(C.byref(bad)) == status, field
    assert L.stp_check_desc(None) == 1


def _stage(n_layers, n_mb, chain_break=None):
    descs = (stp.LayerDesc * n_layers)(*[stp.make_desc(synth.WORKLOADS["tiny"]) for _ in range(n_layers)])
    cb = (C.c_int32 * (n_layers + 1))(*chain_break) if chain_break else None
    return stp.Stage(n_layers=n_layers, n_microbatches=n_mb, desc=descs, chain_break=cb), descs, cb


def _validate(stage, ops):
    arr = (Op * len(ops))(*ops)
    bad = C.c_size_t()
    rc = stp.lib().stp_validate_ops(C.byref(stage), arr, len(ops), C.byref(bad))
    return rc, bad.value


def test_validator_accepts_canonical_sequences():
    from paper_2510_27257_amd.stage import stage_sequence, braid, forward_ops, backward_ops
    for L_, M_ in [(1, 2), (4, 8), (2, 3), (3, 5)]:
        st, *_keep = _stage(L_, M_)
        for step in stage_sequence(L_, M_):
            rc, bad = _validate(st, step)
            assert rc == 0, (L_, M_, bad)
    st, *_keep = _stage(2, 2)
    ops = braid(forward_ops(2, 1), backward_ops(2, 0, OP_BW))
    assert _validate(st, ops) == (0, len(ops))
    # the direction changes at every TP boundary
    kinds = [(o.kind, o.unit) for o in ops[:6]]
    assert kinds == [(OP_F, PRE_ATTN), (OP_F, ATTN), (OP_BW, MLP), (OP_F, PRE_MLP), (OP_F, MLP), (OP_BW, PRE_MLP)]


def test_validator_rejects_bad_sequences():
    st, *_keep = _stage(2, 3)
    ESEQ, EINVAL = 5, 1
    # forward microbatch must exceed the backward microbatch (Appendix A)
    assert _validate(st, [Op(OP_F, PRE_ATTN, 0, 1), Op(OP_B, MLP, 1, 1)]) == (ESEQ, 1)
    assert _validate(st, [Op(OP_F, PRE_ATTN, 0, 1), Op(OP_B, MLP, 1, 2)]) == (ESEQ, 1)
    assert _validate(st, [Op(OP_F, PRE_ATTN, 0, 1), Op(OP_B, MLP, 1, 0)])[0] == 0
    # two forward microbatches in one block
    assert _validate(st, [Op(OP_F, PRE_ATTN, 0, 1), Op(OP_F, ATTN, 0, 2)]) == (ESEQ, 1)
    # forward units out of dependence order
    assert _validate(st, [Op(OP_F, PRE_ATTN, 0, 1), Op(OP_F, PRE_MLP, 0, 1)]) == (ESEQ, 1)
    assert _validate(st, [Op(OP_F, MLP, 0, 1), Op(OP_F, PRE_ATTN, 0, 1)]) == (ESEQ, 1)
    assert _validate(st, [Op(OP_F, MLP, 0, 1), Op(OP_F, PRE_ATTN, 1, 1)])[0] == 0
    # backward units out of order
    assert _validate(st, [Op(OP_B, MLP, 1, 0), Op(OP_B, ATTN, 1, 0)]) == (ESEQ, 1)
    assert _validate(st, [Op(OP_B, PRE_ATTN, 1, 0), Op(OP_B, MLP, 1, 0)]) == (ESEQ, 1)
    assert _validate(st, [Op(OP_B, PRE_ATTN, 1, 0), Op(OP_BW, MLP, 0, 0)])[0] == 0
    # W exists only for Attn and MLP
    assert _validate(st, [Op(OP_W, PRE_MLP, 0, 0)]) == (ESEQ, 0)
    # out-of-range fields
    assert _validate(st, [Op(OP_F, ATTN, 2, 0)]) == (EINVAL, 0)
    assert _validate(st, [Op(7, ATTN, 0, 0)]) == (EINVAL, 0)
    assert _validate(st, [Op(OP_F, ATTN, 0, 3)]) == (EINVAL, 0)
    assert _validate(st, []) == (0, 0)


def test_validator_chain_breaks():
    st, *_keep = _stage(4, 2, chain_break=[0, 0, 1, 0, 0])
    # after the last layer of chain A the next forward op may only start chain B
    assert _validate(st, [Op(OP_F, MLP, 1, 1), Op(OP_F, PRE_ATTN, 2, 1)])[0] == 0
    assert _validate(st, [Op(OP_F, MLP, 1, 1), Op(OP_F, PRE_ATTN, 3, 1)])[0] == 5
    # backward of chain B ends at layer 2; a new backward chain starts at the last layer of a chain
    assert _validate(st, [Op(OP_B, PRE_ATTN, 2, 0), Op(OP_B, MLP, 1, 0)])[0] == 0
    assert _validate(st, [Op(OP_B, PRE_ATTN, 2, 0), Op(OP_B, MLP, 0, 0)])[0] == 5


def test_validator_rejects_chained_layers_of_different_extent():
    """A layer writes its output into the next layer's input slot, so without a chain break the two layer
    descriptions must agree in tokens, hidden size and element type (the ViT -> LM junction of a heterogeneous
    stage needs a chain break)."""
    ESHAPE = 2
    small, big = stp.make_desc(synth.WORKLOADS["tiny"]), stp.make_desc(synth.WORKLOADS["tiny"])
    big.hidden, big.heads_local = 512, 8
    ops = [Op(OP_F, PRE_ATTN, 0, 0)]
    for field, value in [("hidden", 512), ("seq", 256), ("dtype", stp.BF16)]:
        other = stp.make_desc(synth.WORKLOADS["tiny"])
        setattr(other, field, value)
        descs = (stp.LayerDesc * 2)(small, other)
        st = stp.Stage(n_layers=2, n_microbatches=1, desc=descs)
        assert _validate(st, ops)[0] == ESHAPE, field
        cb = (C.c_int32 * 3)(0, 1, 0)
        st = stp.Stage(n_layers=2, n_microbatches=1, desc=descs, chain_break=cb)
        assert _validate(st, ops)[0] == 0, field
    # the same tokens split differently over seq and mbsz chain fine
    other = stp.make_desc(synth.WORKLOADS["tiny"], mbsz=2, seq=64)
    descs = (stp.LayerDesc * 2)(small, other)
    assert _validate(stp.Stage(n_layers=2, n_microbatches=1, desc=descs), ops)[0] == 0


# ---- op-list variants: warm-up depth (Appendix A) and the two pairing patterns of Section 4.1 -------------
def _census(steps):
    """How often each (kind-of-work, unit, layer, microbatch) is issued; BW counts as a B and a W."""
    from collections import Counter
    c = Counter()
    for st in steps:
        for o in st:
            if o.kind == OP_F:
                c[("F", o.unit, o.layer, o.microbatch)] += 1
            if o.kind in (OP_B, OP_BW):
                c[("B", o.unit, o.layer, o.microbatch)] += 1
            if o.kind == OP_W or (o.kind == OP_BW and o.unit in (ATTN, MLP)):
                c[("W", o.unit, o.layer, o.microbatch)] += 1
    return c


def _complete(L_, M_):
    exp = {}
    for l in range(L_):
        for mb in range(M_):
            for u in (PRE_ATTN, ATTN, PRE_MLP, MLP):
                exp[("F", u, l, mb)] = 1
                exp[("B", u, l, mb)] = 1
            for u in (ATTN, MLP):
                exp[("W", u, l, mb)] = 1
    return exp


@pytest.mark.parametrize("warmup", [1, 2, 3, 5])
@pytest.mark.parametrize("n_mb", [3, 4, 6, 8, 12])
def test_warmup_depths_give_valid_complete_sequences(warmup, n_mb):
    from paper_2510_27257_amd.stage import stage_sequence, peak_in_flight
    L_ = 3
    st, *_keep = _stage(L_, n_mb)
    steps = stage_sequence(L_, n_mb, warmup=warmup)
    # the validator carries "B already done" from step to step only inside a context; stand-alone it
    # accepts a W whose B came in an earlier step, and checks everything else
    for step in steps:
        rc, bad = _validate(st, step)
        assert rc == 0, (warmup, n_mb, bad)
    assert dict(_census(steps)) == _complete(L_, n_mb)
    # every W after its B
    seen_b = set()
    for step in steps:
        for o in step:
            if o.kind in (OP_B, OP_BW):
                seen_b.add((o.unit, o.layer, o.microbatch))
            if o.kind == OP_W:
                assert (o.unit, o.layer, o.microbatch) in seen_b
    if n_mb >= warmup + 3:
        # `warmup` plain forward passes come first, and that many more microbatches stay in flight
        assert all(all(o.kind == OP_F for o in s) for s in steps[:warmup])
        assert any(o.kind != OP_F for o in steps[warmup])
        assert peak_in_flight(steps, L_) == L_ * (warmup + 3)


def test_deeper_warmup_keeps_more_stashes_alive():
    from paper_2510_27257_amd.stage import stage_sequence, peak_in_flight
    peaks = [peak_in_flight(stage_sequence(4, 12, warmup=k), 4) for k in (1, 2, 3, 4)]
    assert peaks == sorted(peaks) and len(set(peaks)) == 4
    assert peaks[0] == 16            # F0 .. F3 alive while W0 runs


@pytest.mark.parametrize("pattern", [1, 2])
@pytest.mark.parametrize("n_mb", [1, 2, 3, 6])
@pytest.mark.parametrize("split", [(4, 2), (5, 3), (3, 1)])
def test_two_chunk_patterns_are_valid_and_complete(pattern, n_mb, split):
    from paper_2510_27257_amd.stage import two_chunk_sequence
    L_, first1 = split
    cb = [0] * (L_ + 1)
    cb[first1] = 1
    st, *_keep = _stage(L_, max(n_mb, 1), chain_break=cb)
    steps = two_chunk_sequence(L_, first1, n_mb, pattern)
    for step in steps:
        rc, bad = _validate(st, step)
        assert rc == 0, (pattern, n_mb, split, bad)
    assert dict(_census(steps)) == _complete(L_, n_mb)
    # "V" order per microbatch: forward chunk 0 before chunk 1, backward chunk 1 before chunk 0
    pos = {}
    for si, step in enumerate(steps):
        for o in step:
            pos.setdefault((o.kind == OP_F, o.layer >= first1, o.microbatch), si)
    for mb in range(n_mb):
        assert pos[(True, False, mb)] < pos[(True, True, mb)] < pos[(False, True, mb)] < pos[(False, False, mb)]


def test_the_two_patterns_differ_only_in_the_pairing():
    from paper_2510_27257_amd.stage import two_chunk_sequence
    a, b = two_chunk_sequence(4, 2, 5, 1), two_chunk_sequence(4, 2, 5, 2)
    as_tuples = lambda steps: [[(o.kind, o.unit, o.layer, o.microbatch) for o in st] for st in steps]
    assert _census(a) == _census(b) and as_tuples(a) != as_tuples(b)
    # pattern 2 pairs units of one chunk, pattern 1 of different chunks
    for steps, same in ((b, True), (a, False)):
        for st in steps:
            fc = {o.layer >= 2 for o in st if o.kind == OP_F}
            bc = {o.layer >= 2 for o in st if o.kind != OP_F}
            if fc and bc:
                assert (fc == bc) == same
