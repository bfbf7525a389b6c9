"""The two parity metrics on planted mistakes (CPU only): an error confined to the computed branch of a
residual-carrying output (Eq. 1: branch + X/t, Eq. 2: norm_bwd + dY) passes max|got - ref| / max|ref| when the
residual is large, and fails the residual-subtracted bound."""
import numpy as np

from harness import TOL, STORE_ULP, branch_err, rel_err
from paper_2510_27257_amd import synth


def _case(scale_resid):
    rng = np.random.default_rng(5)
    branch = rng.standard_normal((64, 32)) * 0.05
    resid = rng.standard_normal((64, 32)) * scale_resid
    return branch, resid


def test_branch_metric_catches_what_the_diluted_one_misses():
    branch, resid = _case(8.0)
    ref = branch + resid / 2
    wrong = 2.0 * branch + resid / 2                       # the branch is a factor 2 off
    assert rel_err(wrong, ref) < TOL["bf16"]               # diluted by the residual: passes the plain bound
    assert branch_err(wrong, resid, ref, resid, 0.5, "bf16") > 1.0


def test_branch_metric_accepts_the_rounding_of_the_stored_sum():
    for dtype in ("bf16", "f32"):
        branch, resid = _case(8.0)
        ref = branch + resid / 2
        stored = synth.quantize(ref.astype(np.float32), dtype).astype(np.float64)    # exact branch, one rounding of the sum
        assert branch_err(stored, resid, ref, resid, 0.5, dtype) < 1.0
        assert np.max(np.abs(stored - ref)) <= STORE_ULP[dtype] * np.max(np.abs(ref)) * (1 + 1e-4)   # bf16: the cast to fp32 on the way adds 2^-24


def test_branch_metric_uses_each_side_s_own_residual():
    branch, resid = _case(1.0)
    ref = branch + resid
    resid_path = synth.quantize(resid.astype(np.float32), "bf16").astype(np.float64)  # the path's stored residual input
    got = branch + resid_path
    assert branch_err(got, resid_path, ref, resid, 1.0, "bf16") < 1e-6
