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
