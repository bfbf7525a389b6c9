"""Host-side checks of the schedule generator and simulator (Section 4.2; Table 1)."""
import ctypes as C
import itertools

import pytest

import paper_2510_27257_amd as stp
from paper_2510_27257_amd import schedule as S, synth
from paper_2510_27257_amd.binding import Op, OP_F, OP_B, OP_W, OP_BW

CASES = [(1, 3), (1, 8), (2, 6), (2, 8), (2, 13), (3, 9), (3, 16), (4, 12), (4, 24), (6, 20), (8, 24), (8, 40)]
TIMES = [S.Times(1.0, 1.0, 0.6, 0.25), S.Times(1.0, 2.0, 1.0, 0.5), S.Times(3.0, 3.5, 2.5, 0.0), S.Times(1.0, 1.3, 1.1, 1.0)]


@pytest.mark.parametrize("p,m", CASES)
def test_every_part_runs_exactly_once_on_its_device(p, m):
    for d, prog in enumerate(S.build(p, m)):
        fs = [b.f for b in prog if b.f]
        bs = [b.b for b in prog if b.b]
        ws = [x for b in prog for x in b.w]
        want = sorted(itertools.product((0, 1), range(m)))
        assert sorted(fs) == want and sorted(bs) == want and sorted(ws) == want
        # microbatches of a chunk go through in order, in both directions
        for c in (0, 1):
            assert [i for (cc, i) in fs if cc == c] == list(range(m))
            assert [i for (cc, i) in bs if cc == c] == list(range(m))
        # a W never precedes its B
        seen = set()
        for b in prog:
            if b.b:
                seen.add(b.b)
            assert all(x in seen for x in b.w)


def check_dependencies(p, progs, t, flow="v", atomic_bw=False):
    """Independent of the simulator's bookkeeping: every start respects the results it needs."""
    V = 2 * p
    vstage = lambda p_, d_, c_: S.vstage(p_, d_, c_, flow)
    f_done, b_done, pos = {}, {}, {}
    for d, prog in enumerate(progs):
        prev_end = 0.0
        for blk in prog:
            assert blk.start >= prev_end - 1e-9
            dur = (t.TF if blk.f else 0) + (t.TB if blk.b else 0) + len(blk.w) * t.TW
            alone = (blk.f is None) != (blk.b is None) and not blk.w
            assert abs(blk.end - blk.start - dur - (t.TAR if alone else 0)) < 1e-9
            prev_end = blk.end
            if blk.f and blk.b:
                out = blk.start + t.TF + t.TB
            elif blk.f:
                out = blk.start + t.TF + (t.TAR if alone else 0)
            else:
                out = blk.start + t.TB + (t.TAR if alone else 0) + (t.TW if atomic_bw and blk.b in blk.w else 0)
            if blk.f:
                f_done[(vstage(p, d, blk.f[0]), blk.f[1])] = out
            if blk.b:
                b_done[(vstage(p, d, blk.b[0]), blk.b[1])] = out
    for d, prog in enumerate(progs):
        for blk in prog:
            if blk.f:
                v, i = vstage(p, d, blk.f[0]), blk.f[1]
                if v > 0:
                    assert blk.start >= f_done[(v - 1, i)] - 1e-9
            if blk.b:
                v, j = vstage(p, d, blk.b[0]), blk.b[1]
                assert blk.start >= f_done[(v, j)] - 1e-9
                if v < V - 1:
                    assert blk.start >= b_done[(v + 1, j)] - 1e-9
            for x in blk.w:
                if x != blk.b:
                    assert blk.start >= b_done[(vstage(p, d, x[0]), x[1])] - 1e-9


@pytest.mark.parametrize("p,m", CASES)
@pytest.mark.parametrize("t", TIMES)
def test_simulated_programs_respect_every_dependency(p, m, t):
    progs = S.build(p, m)
    T = S.simulate(p, progs, t)
    check_dependencies(p, progs, t)
    assert abs(T - max(b.end for pr in progs for b in pr)) < 1e-9
    # same blocks after W blocks floated into waits
    for d, prog in enumerate(progs):
        assert sorted(x for b in prog for x in b.w) == sorted(itertools.product((0, 1), range(m)))


@pytest.mark.parametrize("p,m", CASES)
@pytest.mark.parametrize("t", TIMES)
def test_table1_tp_bubble_and_peak_activation_memory(p, m, t):
    """Table 1, row of the proposed schedule: non-overlapped TP communication (2p+1) T_AR on every device, peak
    activation memory 3p M_a (device 0; device d holds 3p - d), and the start-up part of the PP bubble."""
    progs = S.build(p, m)
    S.simulate(p, progs, t)
    ms = S.metrics(p, progs, t)
    ref = S.table1(p, t)
    for d, x in enumerate(ms):
        assert abs(x["tp_bubble"] - ref["tp_bubble"]) < 1e-9
        assert x["peak_activation"] == 3 * p - d
        assert abs(x["start_idle"] - d * (t.TF + t.TAR)) < 1e-9
        assert x["peak_with_w_stash"] >= x["peak_activation"]
    assert ms[0]["peak_activation"] == ref["peak_activation"]
    # every device waits the same total time, and never less than Table 1's (approximate) PP bubble
    # (test_pp_bubble_against_table1_and_its_floor looks at what the difference is made of)
    assert max(x["pp_bubble"] for x in ms) - min(x["pp_bubble"] for x in ms) < 1e-6
    assert ms[0]["pp_bubble"] >= ref["pp_bubble"] - 1e-9


def test_pp_bubble_against_table1_and_its_floor():
    """Table 1 gives the PP bubble of the proposed schedule as approximately (p-1)(T_F + T_AR + T_B - T_W).  Its
    first part, (p-1)(T_F + T_AR), is a floor for ANY schedule: the last device cannot start before the first
    microbatch has crossed p-1 stages, every device is busy for the same time, so nobody waits less in total.  The
    construction here (made from the text; the schedule figure is not in it) meets that floor exactly at the start
    of the last device, does not depend on the number of microbatches, and with no weight-gradient separation in
    the steady phase stays above the closed form (at most 2.5 times): its excess sits in the last device's wait
    for the first gradient to come round and in the cool-down, which only stored weight-gradient blocks can fill.
    Storing the W of the last steady braids (steady_w_tail) never makes it larger and never brings it below the
    closed form (it comes within 6 % of it for T_AR = T_F)."""
    for t in TIMES:
        for p in (2, 3, 4, 8):
            bubbles = []
            for m in (3 * p, 3 * p + 5, 6 * p):
                progs = S.build(p, m)
                S.simulate(p, progs, t)
                ms = S.metrics(p, progs, t)
                floor = (p - 1) * (t.TF + t.TAR)
                assert abs(ms[p - 1]["start_idle"] - floor) < 1e-9
                assert all(x["pp_bubble"] >= floor - 1e-9 for x in ms)
                bubbles.append(ms[0]["pp_bubble"])
            assert max(bubbles) - min(bubbles) < 1e-6               # the bubble is a property of p and the times only
            ref = S.table1(p, t)["pp_bubble"]
            assert ref - 1e-9 <= bubbles[0] <= 2.5 * ref
            for tail in (p, 2 * p):
                progs = S.build(p, 6 * p, steady_w_tail=tail)
                S.simulate(p, progs, t)
                b = S.metrics(p, progs, t)[0]["pp_bubble"]
                assert ref - 1e-9 <= b <= bubbles[0] + 1e-9
                prev = b


ROW_CASES = [(1, 3), (2, 8), (3, 9), (4, 12), (4, 24), (8, 24), (8, 40)]


@pytest.mark.parametrize("p,m", ROW_CASES)
@pytest.mark.parametrize("t", TIMES)
def test_table1_row_of_interleaved_1f1b(p, m, t):
    """Table 1, row 1F1B-I (two virtual stages, parallel flow, unsplit backward): the simulated programs give the PP
    bubble (p-1)(T_F + T_AR + T_B + T_W) and the TP bubble 2 m T_AR exactly, on every device; the activations alive
    on device d peak at 3p - 2 - 2d before the steady phase (the table's figure for device 0) plus the one forward
    pass of a steady pair that runs before its backward pass frees a slot."""
    progs = [S.program_1f1b_interleaved(p, m, d) for d in range(p)]
    want = sorted(itertools.product((0, 1), range(m)))
    for prog in progs:
        assert sorted(b.f for b in prog if b.f) == want and sorted(b.b for b in prog if b.b) == want
        assert all(b.w == (b.b,) for b in prog if b.b) and all(not b.w for b in prog if b.f)
    S.simulate(p, progs, t, float_w=False, flow="parallel", atomic_bw=True)
    check_dependencies(p, progs, t, flow="parallel", atomic_bw=True)
    ref = S.table1(p, t, "1f1b-i", m)
    for d, x in enumerate(S.metrics(p, progs, t)):
        assert abs(x["pp_bubble"] - ref["pp_bubble"]) < 1e-6
        assert abs(x["tp_bubble"] - ref["tp_bubble"]) < 1e-9
        warm = min(2 * (p - d - 1) + p, 2 * m)
        assert x["peak_activation"] == min(warm + 1, 2 * m)
    assert min(2 * (p - 1) + p, 2 * m) == min(ref["peak_activation"], 2 * m)


@pytest.mark.parametrize("p,m", ROW_CASES)
@pytest.mark.parametrize("t", TIMES)
def test_table1_row_of_zero_bubble_v(p, m, t):
    """Table 1, row ZB-V, from a list-scheduled program (forward, activation-gradient and weight-gradient passes all
    separate, "V" flow, at most 2p chunk-activations alive): TP bubble 4 m T_AR and peak activation memory 2p as
    in the table.  The PP bubble of this greedy program is above the table's (p-1)(T_F + 2 T_AR + T_B - 2 T_W),
    which belongs to a hand-made schedule: unpinned."""
    progs = S.greedy_zero_bubble_v(p, m, t)
    want = sorted(itertools.product((0, 1), range(m)))
    for prog in progs:
        assert sorted(b.f for b in prog if b.f) == want and sorted(b.b for b in prog if b.b) == want
        assert sorted(x for b in prog for x in b.w) == want
        assert all(sum(map(bool, (b.f, b.b, b.w))) == 1 for b in prog)
    check_dependencies(p, progs, t)
    ref = S.table1(p, t, "zb-v", m)
    for x in S.metrics(p, progs, t):
        assert abs(x["tp_bubble"] - ref["tp_bubble"]) < 1e-9
        assert x["peak_activation"] == min(ref["peak_activation"], 2 * m)
        assert x["pp_bubble"] >= min(ref["pp_bubble"], (p - 1) * (t.TF + t.TAR)) - 1e-9


@pytest.mark.parametrize("p,m", [(2, 8), (4, 12), (4, 24), (8, 24), (8, 40)])
def test_with_tp_communication_the_proposed_schedule_finishes_first(p, m):
    """The comparison of Section 5 in the simulator: once the all-reduce time is a sizeable part of a chunk's
    forward time, the proposed schedule finishes before interleaved 1F1B, and Zero Bubble V, which exposes the
    all-reduce of every forward and every backward pass, is the slowest of the three."""
    for t in (S.Times(1.0, 1.0, 0.6, 0.25), S.Times(1.0, 2.0, 1.0, 0.5), S.Times(1.0, 1.3, 1.1, 1.0)):
        ours = S.build(p, m)
        T_ours = S.simulate(p, ours, t)
        i1 = [S.program_1f1b_interleaved(p, m, d) for d in range(p)]
        T_1f1b = S.simulate(p, i1, t, float_w=False, flow="parallel", atomic_bw=True)
        T_zbv = max(b.end for pr in S.greedy_zero_bubble_v(p, m, t) for b in pr)
        assert T_ours < T_1f1b < T_zbv


def test_simulator_on_a_case_worked_by_hand():
    """One device (p = 1: virtual stages 0 and 1), three microbatches, T_F = 1, T_B = 2, T_W = 1, T_AR = 0.5: the
    2p+1 = 3 warm-up forward passes are the only blocks with an exposed all-reduce, and a lone device never
    waits, so the makespan is all the work plus three all-reduces."""
    t = S.Times(1.0, 2.0, 1.0, 0.5)
    progs = S.build(1, 3)
    names = [b.name() for b in progs[0]]
    assert names[:3] == ["F0.0", "F1.0", "F0.1"]
    T = S.simulate(1, progs, t)
    # one device never waits for another: the makespan is the sum of its blocks
    plain = sum(1 for b in progs[0] if (b.f is None) != (b.b is None) and not b.w)
    assert plain == 3
    assert abs(T - (2 * 3 * (1.0 + 2.0 + 1.0) + 3 * 0.5)) < 1e-9
    assert S.metrics(1, progs, t)[0]["pp_bubble"] < 1e-9


def test_two_devices_first_blocks_by_hand():
    """p = 2, unit times, no all-reduce: device 1 starts one forward later; device 0's first chunk-1 forward can
    start when microbatch 0 has passed virtual stages 1 and 2 on device 1 (t = 3), its first backward follows."""
    t = S.Times(1.0, 1.0, 1.0, 0.0)
    progs = S.build(2, 6)
    S.simulate(2, progs, t)
    d0, d1 = progs
    assert [b.name() for b in d0[:6]] == ["F0.0", "F0.1", "F0.2", "F1.0", "F0.3", "F1.1&B1.0"]
    assert [b.start for b in d0[:6]] == [0.0, 1.0, 2.0, 3.0, 4.0, 5.0]
    assert [b.name() for b in d1[:5]] == ["F0.0", "F1.0", "F0.1", "F1.1", "F0.2"]
    assert [b.start for b in d1[:5]] == [1.0, 2.0, 3.0, 4.0, 5.0]
    # the last device never separates W in the warm-up; device 0 does, once (p - d - 1 = 1), and uses it at once
    assert d0[6].name() == "F0.4&W1.0"
    assert d1[5].name() == "F1.2&BW1.0"


@pytest.mark.parametrize("p,m", [(2, 8), (3, 16), (4, 16), (4, 24), (8, 40)])
@pytest.mark.parametrize("t", TIMES)
def test_weight_separation_late_in_the_steady_phase(p, m, t):
    """Section 4.2: separation in the steady phase trades stash memory for bubbles.  Storing the W of the last
    braids of the phase leaves every part in place once, breaks no dependency, keeps Table 1's TP bubble and peak
    activation memory, never lengthens the step, and holds more W stashes."""
    base = S.build(p, m)
    T0 = S.simulate(p, base, t)
    m0 = S.metrics(p, base, t)
    for tail in (1, p, 2 * p):
        progs = S.build(p, m, steady_w_tail=tail)
        for d, prog in enumerate(progs):
            want = sorted(itertools.product((0, 1), range(m)))
            assert sorted(b.f for b in prog if b.f) == want and sorted(b.b for b in prog if b.b) == want
            assert sorted(x for b in prog for x in b.w) == want
        T = S.simulate(p, progs, t)
        check_dependencies(p, progs, t)
        ms = S.metrics(p, progs, t)
        ref = S.table1(p, t)
        for d, x in enumerate(ms):
            assert abs(x["tp_bubble"] - ref["tp_bubble"]) < 1e-9
            assert x["peak_activation"] == 3 * p - d
            assert x["peak_with_w_stash"] >= m0[d]["peak_with_w_stash"]
        assert T <= T0 + 1e-9
        assert ms[0]["pp_bubble"] >= ref["pp_bubble"] - 1e-9


def test_too_few_microbatches_are_refused():
    with pytest.raises(ValueError):
        S.device_program(4, 11, 0)
    with pytest.raises(ValueError):
        S.device_program(2, 8, 2)


def _stage(n_layers, n_mb, chain_break):
    descs = (stp.LayerDesc * n_layers)(*[stp.make_desc(synth.WORKLOADS["tiny"]) for _ in range(n_layers)])
    cb = (C.c_int32 * (n_layers + 1))(*chain_break)
    return stp.Stage(n_layers=n_layers, n_microbatches=n_mb, desc=descs, chain_break=cb), descs, cb


@pytest.mark.parametrize("p,m", [(1, 4), (2, 7), (3, 9), (4, 13)])
def test_the_library_accepts_every_device_program(p, m):
    """A device's program as braid steps over a two-chunk stage passes the library's own validator."""
    t = S.Times(1.0, 1.2, 0.8, 0.3)
    progs = S.build(p, m)
    S.simulate(p, progs, t)
    L, first1 = 3, 2
    st, *_keep = _stage(L, m, [0, 0, 1, 0])
    for d in range(p):
        steps = S.braid_steps(progs[d], L, first1)
        assert len(steps) == len(progs[d])
        n_ops = 0
        for step in steps:
            arr = (Op * len(step))(*step)
            bad = C.c_size_t()
            assert stp.lib().stp_validate_ops(C.byref(st), arr, len(step), C.byref(bad)) == 0, (d, bad.value)
            n_ops += len(step)
        # 4 F units, 4 B units and 2 W units per layer and microbatch; a BW op stands for a B and a W
        f = sum(1 for s in steps for o in s if o.kind == OP_F)
        b = sum(1 for s in steps for o in s if o.kind in (OP_B, OP_BW))
        w = sum(1 for s in steps for o in s if o.kind == OP_W or (o.kind == OP_BW and o.unit in (1, 3)))
        assert (f, b, w) == (4 * L * m, 4 * L * m, 2 * L * m)
