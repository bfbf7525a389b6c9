"""Host-side checks of the tile tuning helpers (no GPU): the GEMM shapes of a layer as the units call them, the
coordinate descent on a synthetic objective, and the stored table."""
import json

from paper_2510_27257_amd import synth, tune


class FakeCtx:
    def __init__(self):
        self.hints = {}

    def gemm_tile_hint(self, M, N, K, at, bt, tm, tn):
        if tm == 0 and tn == 0:
            self.hints.pop((M, N, K, at, bt), None)
        else:
            self.hints[(M, N, K, at, bt)] = (tm, tn)

    def gemm_tile_hints_clear(self):
        self.hints.clear()


def test_layer_gemm_shapes_cover_the_units_of_section_3():
    wl = synth.WORKLOADS["gpt7b_tp8"]
    s = tune.layer_gemm_shapes(wl)
    T, h, a, f, q = wl.seq, wl.hidden, wl.attn_local, wl.ffn_local, wl.qkv_local
    # forward: activations [T, in] times weights [in, out]; B: the weight read transposed; W: contraction over tokens
    assert s["qkv_f"] == (T, q, h, 0, 0) and s["fc2_f"] == (T, h, f, 0, 0)
    assert s["out_b"] == (T, a, h, 0, 1) and s["fc2_b"] == (T, f, h, 0, 1)
    assert s["fc1_w"] == (h, f, T, 1, 0) and s["out_w"] == (a, h, T, 1, 0)
    # the same flops forwards, backwards and for the weights: 2 M N K agrees per linear layer
    for lin in ("qkv", "out", "fc1", "fc2"):
        vols = {k[-1]: v[0] * v[1] * v[2] for k, v in s.items() if k.startswith(lin)}
        assert len(set(vols.values())) == 1, lin
    assert len(s) == 12


def test_descent_finds_the_planted_preferences_and_nothing_else():
    ctx = FakeCtx()
    shapes = tune.layer_gemm_shapes(synth.WORKLOADS["tiny"])
    want = {shapes["fc1_w"]: (256, 256), shapes["out_b"]: (128, 256)}

    def run():          # a block that is 3 % faster for each planted preference that is in place, 1 % slower for others
        ms = 1.0
        for shape, tile in ctx.hints.items():
            ms *= 0.97 if want.get(shape) == tile else 1.01
        return ms

    hints, base, final = tune.descend(ctx, shapes, run)
    assert base == 1.0 and abs(final - 0.97 ** 2) < 1e-12
    assert hints == {",".join(map(str, k)): f"{v[0]}x{v[1]}" for k, v in want.items()}
    assert ctx.hints == want                      # what stays in the context is what is reported


def test_descent_drops_a_set_that_does_not_beat_the_library_choice_in_the_end():
    ctx = FakeCtx()
    shapes = tune.layer_gemm_shapes(synth.WORKLOADS["tiny"])
    calls = {"n": 0}

    def run():          # drift: every measurement a little faster than the one before, whatever the tiles are
        calls["n"] += 1
        return 1.0 * 0.999 ** calls["n"]

    hints, base, final = tune.descend(ctx, shapes, run, passes=1)
    assert hints == {} and ctx.hints == {} and base == final


def test_stored_tables_are_well_formed_and_apply(tmp_path):
    for objective in ("block", "stage"):
        table = tune.load_hints(objective=objective)
        assert table, objective
        for name, hints in table.items():
            assert name in synth.WORKLOADS
            shapes = set(tune.layer_gemm_shapes(synth.WORKLOADS[name]).values())
            for key, tile in hints.items():
                assert tuple(int(v) for v in key.split(",")) in shapes, (name, key)     # a GEMM this workload really runs
                assert tile in ("256x256", "128x256", "256x128", "128x128") or (tile == "192x256" and key.split(",")[3] == "0")
    p = tmp_path / "t.json"
    p.write_text(json.dumps({"workloads": {"gpt7b_tp8": {"8,16,24,1,0": "128x256"}},
                             "stage_workloads": {"gpt7b_tp8": {}, "vit": {"8,16,24,0,0": "256x128"}}}))
    ctx = FakeCtx()
    assert tune.apply_tuned(ctx, ["gpt7b_tp8", "vit", "gpt7b_tp8"], str(p)) == ["gpt7b_tp8"]
    assert ctx.hints == {(8, 16, 24, 1, 0): (128, 256)}
    ctx = FakeCtx()             # the other objective has a table of its own; an empty entry counts as an entry
    assert tune.apply_tuned(ctx, ["gpt7b_tp8", "vit"], str(p), objective="stage") == ["gpt7b_tp8", "vit"]
    assert ctx.hints == {(8, 16, 24, 0, 0): (256, 128)}
    assert tune.load_hints(str(tmp_path / "absent.json")) == {}
    try:
        tune.load_hints(objective="layer")
        assert False
    except ValueError:
        pass
