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


def check_layers(ovf, pipe, space, model, w, cids, vals, states, tol, layers=None, eps=0.0, seed=0, rollout=0):
    """A schedule of the GPU against the checker, decision by decision, each under the GPU's own
    committed prefix.  For every layer looked at: the GPU's choice must be a valid candidate; by
    the checker's scores (exploration noise of `rollout` included) it must be the first minimum,
    or lie within the tolerance of it - (score of the GPU's choice - minimum) / max(|minimum|,
    RMS of the valid scores) <= tol - and the GPU's value must agree with the checker's score of
    that same candidate.  All state records must be what the chosen ids replay to.  Returns the
    number of decisions that differed inside the margin."""
    cids = np.asarray(cids); vals = np.asarray(vals)
    S = len(pipe)
    layers = range(S) if layers is None else layers
    n_margin = 0
    for i in layers:
        assert (cids[:i] >= 0).all(), "layer behind the end of the schedule"
        sc, ok = ovf.decision_scores(pipe, space, model, w, cids[:i], i, eps, seed, rollout)
        sc = sc.astype(np.float64)
        cand = np.flatnonzero(ok & (sc < np.inf))
        if len(cand) == 0:
            assert cids[i] == -1 and vals[i] == np.inf, f"layer {i}: a winner where the checker has none"
            continue
        best = int(cand[np.argmin(sc[cand])])
        g = int(cids[i])
        assert g >= 0 and ok[g], f"layer {i}: GPU chose an invalid candidate ({g})"
        s = max(float(np.sqrt(np.mean(sc[cand] ** 2))), 1e-30)
        if g != best:
            margin = (sc[g] - sc[best]) / max(abs(sc[best]), s)
            assert margin <= tol, f"layer {i}: decision {g} vs {best} differs outside the margin ({margin})"
            n_margin += 1
        err = abs(float(vals[i]) - sc[g]) / max(abs(sc[g]), s)
        assert err <= tol, f"layer {i}: value of candidate {g} off by {err}"
    if states is not None:
        n = int(np.argmax(cids < 0)) if (cids < 0).any() else S
        rst, _ = ovf.states(pipe, space, cids[:n])
        assert np.array_equal(rst, np.asarray(states)[:n]), "state records are not what the ids replay to"
        assert not np.asarray(states)[n:].any()
    return n_margin
