"""Helpers shared by the GPU parity tests."""
import numpy as np

TOL = {0: 1e-5, 1: 2e-2}  # fp32 path, bf16 path (scale-relative, see score_err)


def score_err(got, ref):
    """|got - ref| / max(|ref|, s), s = RMS of the finite reference scores: scores of a
    random-weight network straddle zero, so a plain relative error is ill-posed."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    fin = np.isfinite(ref)
    assert np.array_equal(fin, np.isfinite(got)), "finite / non-finite pattern differs"
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    assert np.array_equal(ref[~fin & ~np.isnan(ref)], got[~fin & ~np.isnan(ref)])
    if not fin.any():
        return 0.0
    s = max(float(np.sqrt(np.mean(ref[fin] ** 2))), 1e-30)
    return float(np.max(np.abs(got[fin] - ref[fin]) / np.maximum(np.abs(ref[fin]), s)))


def check_argmin(gpu_idx, gpu_val, ref_scores, valid, tol, lo=0):
    """The GPU winner must be the checker's first minimum unless the checker's top-2
    margin is below the tolerance; then any candidate within the margin is accepted."""
    ref_scores = np.asarray(ref_scores, np.float64)
    ok = np.ones(len(ref_scores), bool) if valid is None else (np.asarray(valid) != 0)
    cand = np.flatnonzero(ok & (ref_scores < np.inf))
    if len(cand) == 0:
        assert gpu_idx == -1 and gpu_val == np.inf
        return True
    best = cand[np.argmin(ref_scores[cand])]
    if gpu_idx - lo == best:
        return True
    fin = ref_scores[cand]
    s = max(float(np.sqrt(np.mean(fin ** 2))), 1e-30)
    vmin = ref_scores[best]
    assert gpu_idx - lo in set(cand.tolist()), "GPU chose an invalid candidate"
    margin = (ref_scores[gpu_idx - lo] - vmin) / max(abs(vmin), s)
    assert margin <= tol, f"decision differs outside the margin: {gpu_idx - lo} vs {best}, margin {margin}"
    return False
