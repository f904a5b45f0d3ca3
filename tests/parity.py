"""Shared pieces of the GPU parity tests: the stored oracle outputs, the bounds derived from the oracle's stored
self-drift, and the report of measured errors."""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TOL = 2e-2
RMS_FACTOR, MAX_FACTOR = 1.5, 2.0


def report(line):
    """Measured figures: printed, and appended to parity_errors.txt in the run's output folder (PARITY_REPORT_DIR,
    by default the untracked output folder at the repository root) when that folder exists."""
    print(line, flush=True)
    out = os.environ.get("PARITY_REPORT_DIR", os.path.join(os.path.dirname(GOLD), "..", "gpurun_out"))
    if os.path.isdir(out):
        with open(os.path.join(out, "parity_errors.txt"), "a") as f:
            f.write(line + "\n")


def rms(a):
    return float(np.sqrt(np.mean(np.square(a))))


def draft_tolerances(g, depth):
    """(near-tie margin, allowed score error per level) from the oracle's stored self-drift of the scores: the
    per-level figures are maxima over a level's candidates, so the factor for maxima applies."""
    per_level = np.maximum(1e-2, MAX_FACTOR * np.asarray(g["draft_drift_all_per_level"], dtype=np.float64))
    assert len(per_level) == depth
    return float(max(1e-2, np.max(g["draft_drift_all_per_level"]))), per_level


def bounded(name, got, ref, drift, scale=1.0):
    """RMS and max of (got - ref) against the stored self-drift [max, rms]; never tighter than TOL * scale."""
    d = got - ref
    err_max, err_rms = float(np.max(np.abs(d))), rms(d)
    bound_max = max(MAX_FACTOR * float(drift[0]), TOL * scale)
    bound_rms = max(RMS_FACTOR * float(drift[1]), TOL * scale / 4)
    report(f"{name}: max err {err_max:.5f} (bound {bound_max:.5f}, self-drift {float(drift[0]):.5f}); "
            f"rms err {err_rms:.5f} (bound {bound_rms:.5f}, self-drift {float(drift[1]):.5f}); ref rms {rms(ref):.3f}")
    assert err_max <= bound_max, name
    assert err_rms <= bound_rms, name
    return bound_max


def check_scores(tag, got, ref, per_level_tol):
    """Cumulative log-probabilities per level against the oracle's stored score drift of that level."""
    err = np.abs(got["pool_score"] - ref["pool_score"])
    worst = [float(err[ref["pool_depth"] == l + 1].max()) for l in range(len(per_level_tol))]
    report(f"{tag} draft: score error per level {np.round(worst, 5).tolist()}, allowed {np.round(per_level_tol, 5).tolist()}, "
            f"min selection gap {ref['min_gap']:.2e}, near-ties followed {ref['n_followed']}")
    assert np.all(np.asarray(worst) <= per_level_tol)
    assert np.all(np.abs(got["score"] - ref["score"]) <= per_level_tol[np.maximum(ref["depth"], 1) - 1])


def golden(name):
    path = os.path.join(GOLD, f"{name}_verify.npz")
    if not os.path.exists(path):
        pytest.skip(f"{path} not generated (python tests/golden/make_golden.py {name})")
    g = np.load(path)
    if not any(k.endswith("drift_all_logits") for k in g.files):
        pytest.skip(f"{path} predates the self-drift statistics: regenerate it with tests/golden/make_golden.py {name}")
    return g


