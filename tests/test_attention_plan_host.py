"""Host-side checks of the work plan of the chunked attention kernels (no GPU): the plan covers every step of every
block exactly once, in chunks of at most chunk_steps, at most 8 per block, dispatched longest first."""
import heapq

import pytest

import paper_2510_27257_amd as stp
from paper_2510_27257_amd.synth import WORKLOADS, Workload

SHAPES = {
    "gpt7b_tp8": WORKLOADS["gpt7b_tp8"],
    "gpt7b_tp8_s4096": WORKLOADS["gpt7b_tp8_s4096"],
    "llama13b_tp4": WORKLOADS["llama13b_tp4"],
    "gqa12b_tp4": WORKLOADS["gqa12b_tp4"],
    "vit": WORKLOADS["vit"],
    "ragged": Workload("r", 512, 4, 128, 1024, 1000, 8),
    "one_block": Workload("o", 256, 2, 128, 512, 72, 8),
    "long": Workload("l", 1024, 8, 128, 1024, 16384, 8),
    "bidirectional_long": Workload("b", 1024, 8, 128, 1024, 8192, 8, causal=False),
}


def steps_of(wl, kind):
    """Steps per block, from the kernels' geometry: 128-row blocks; 128-key steps (forward, dq) or 64-query steps (dkv)."""
    seq, causal = wl.seq, wl.causal
    nb = (seq + 127) // 128
    if kind == stp.ATTN_DKV:
        nq = (seq + 63) // 64
        kv_heads = wl.kv_heads or wl.heads_local
        group = wl.heads_local // kv_heads
        return [group * (nq - (2 * x if causal else 0)) for x in range(nb)]
    return [(min(seq, 128 * (x + 1)) + 127) // 128 if causal else nb for x in range(nb)]


@pytest.mark.parametrize("name", list(SHAPES))
@pytest.mark.parametrize("kind", [stp.ATTN_FWD, stp.ATTN_DKV, stp.ATTN_DQ])
def test_plan_covers_every_step_once_longest_first(name, kind):
    wl = SHAPES[name]
    desc = stp.make_desc(wl)
    c, max_chunks, items = stp.attention_plan(desc, kind)
    steps = steps_of(wl, kind)
    assert c >= 1 and 1 <= max_chunks <= 8
    assert max_chunks == max((s + c - 1) // c for s in steps)
    want = {(x, k) for x, s in enumerate(steps) for k in range((s + c - 1) // c)}
    if len(want) > 1024:
        assert items == []          # the kernel falls back to its blocks x chunks grid
        return
    assert len(items) == len(want) and set(items) == want
    lens = [min(c, steps[x] - k * c) for x, k in items]
    assert all(n >= 1 for n in lens)
    assert lens == sorted(lens, reverse=True)
    assert sum(lens) == sum(steps)


def makespan(lens, z, fixed, per, cus=256):
    free = [0.0] * cus
    heapq.heapify(free)
    end = 0.0
    for n in lens:
        for _ in range(z):
            t = heapq.heappop(free) + fixed + per * n
            end = max(end, t)
            heapq.heappush(free, t)
    return end


@pytest.mark.parametrize("name", ["gpt7b_tp8", "gpt7b_tp8_s4096", "llama13b_tp4"])
def test_planned_chunk_is_no_worse_than_the_former_constant(name):
    """Under the plan's own cost model the chosen chunk length beats (or equals) the constant 16 steps that the
    forward kernel used before, dispatched in the same longest-first order."""
    wl = SHAPES[name]
    desc = stp.make_desc(wl)
    c, _, items = stp.attention_plan(desc, stp.ATTN_FWD)
    steps = steps_of(wl, stp.ATTN_FWD)

    def lens_for(cc):
        out = []
        for s in steps:
            out += [cc] * (s // cc) + ([s % cc] if s % cc else [])
        return sorted(out, reverse=True)

    z = wl.heads_local
    assert makespan(lens_for(c), z, 11.5, 1.75) <= makespan(lens_for(min(16, max(steps))), z, 11.5, 1.75) * 1.005


def test_plan_rejects_bad_arguments():
    import ctypes as C
    desc = stp.make_desc(WORKLOADS["gpt7b_tp8"])
    a, b, n = C.c_int32(), C.c_int32(), C.c_int32()
    L = stp.lib()
    assert L.stp_attention_plan(C.byref(desc), 3, C.byref(a), C.byref(b), C.byref(n), None, 0) == 1      # STP_EINVAL
    assert L.stp_attention_plan(C.byref(desc), 0, None, C.byref(b), C.byref(n), None, 0) == 1
    assert L.stp_attention_plan(C.byref(desc), 0, C.byref(a), C.byref(b), C.byref(n), None, 0) == 0 and n.value > 0
    small = (C.c_uint16 * 4)()
    assert L.stp_attention_plan(C.byref(desc), 0, C.byref(a), C.byref(b), C.byref(n), small, 4) == 4      # STP_ENOSPACE
    f32 = stp.make_desc(WORKLOADS["tiny"])
    assert L.stp_attention_plan(C.byref(f32), 0, C.byref(a), C.byref(b), C.byref(n), None, 0) == 6        # STP_EUNSUPPORTED


def test_plan_invariants_on_random_shapes():
    """Seeded random shapes (sequence length, head counts, grouping, causal or not): the same invariants."""
    import random
    rng = random.Random(20251027)
    for _ in range(60):
        seq = rng.choice([8, 64, 72, 128, 136, 1000, 2048, 4096, 5000, 12288]) if rng.random() < 0.6 else 8 * rng.randint(1, 2500)
        nk = rng.choice([1, 2, 4, 8])
        group = rng.choice([1, 1, 2, 5])
        heads = nk * group
        wl = Workload("r", 512, heads, rng.choice([64, 128]), 512, seq, 8, causal=rng.random() < 0.7, kv_heads=nk if group > 1 else 0)
        desc = stp.make_desc(wl, mbsz=rng.choice([1, 1, 2]))
        for kind in (stp.ATTN_FWD, stp.ATTN_DKV, stp.ATTN_DQ):
            c, max_chunks, items = stp.attention_plan(desc, kind)
            steps = steps_of(wl, kind)
            assert c >= 1 and 1 <= max_chunks <= 8, (seq, heads, nk, kind)
            assert max_chunks == max((s + c - 1) // c for s in steps)
            want = {(x, k) for x, s in enumerate(steps) for k in range((s + c - 1) // c)}
            if len(want) > 1024:
                assert items == []
                continue
            assert len(items) == len(want) and set(items) == want
            lens = [min(c, steps[x] - k * c) for x, k in items]
            assert lens == sorted(lens, reverse=True) and sum(lens) == sum(steps)
