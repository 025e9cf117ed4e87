"""GPU parity: beam search guided by V against the CPU checker."""
import numpy as np
import pytest

from paper_2011_14486_amd import inputs as I
from tests.util import TOL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def vf():
    import paper_2011_14486_amd as pkg
    return pkg.load()


def layer_scores(ovf, pipe, sp, model, w, pre, i):
    """The checker's V of every candidate state of decision i after prefix `pre`:
    (scores float64 [M], valid [M]) for either kind of value network."""
    M = ovf.dense_count(sp)
    if model[0] == I.LSTM:
        x, valid = ovf.sequences(pipe, sp, list(pre), i)
        sc = np.full(M, np.inf)
        ids = np.flatnonzero(valid)
        if len(ids):
            sc[ids] = ovf.score_lstm(model, w, x[ids])
        return sc, valid.astype(bool)
    feat = ovf.featurize(pipe, sp, list(pre), i)
    return ovf.score_mlp(model, w, feat, M=M).astype(np.float64), feat[16, :M] != 0


def check_beam(ovf, pipe, sp, model, w, run, K, tol):
    """Layer by layer (run(last) = the GPU search stopped after layer `last`): the checker
    scores every extension of the GPU's survivors of the layer before; the GPU's survivors
    of this layer must be the smallest ones (up to the score tolerance at the cut), in
    order, with matching values and state records."""
    S = len(pipe)
    prev, vals_prev = [()], [np.zeros(0, np.float32)]
    for i in range(S):
        cids, vals, states, n_beams = run(i)
        items = []
        for b, pre in enumerate(prev):
            sc, valid = layer_scores(ovf, pipe, sp, model, w, pre, i)
            for c in np.flatnonzero(valid):
                if sc[c] < np.inf:
                    items.append((sc[c], b, int(c)))
        items.sort()
        if not items:
            # dead end: the survivors of the layer before are kept as they were
            assert n_beams == len(prev) or (prev == [()] and n_beams == 1)
            for j, pre in enumerate(prev):
                assert tuple(int(t) for t in cids[j, :i]) == pre and (cids[j, i:] == -1).all()
            return
        rows = [j for j in range(K) if cids[j, i] >= 0]
        assert rows == list(range(len(rows))) and len(rows) == min(K, len(items)) == n_beams
        score_of = {(b, c): s for s, b, c in items}
        scale = max(float(np.sqrt(np.mean([s * s for s, _, _ in items]))), 1e-30)
        got = []
        for j in rows:
            pre = tuple(int(t) for t in cids[j, :i])
            assert pre in prev, f"layer {i}: row {j} does not extend a survivor of the layer before"
            key = (prev.index(pre), int(cids[j, i]))
            assert key in score_of, f"layer {i}: row {j} is not a valid candidate"
            got.append((score_of[key], key))
            err = abs(float(vals[j, i]) - score_of[key]) / max(abs(score_of[key]), scale)
            assert err <= tol, (i, j, err)
            assert np.array_equal(vals[j, :i], vals_prev[key[0]][:i])
            rst, _ = ovf.states(pipe, sp, cids[j, :i + 1])
            assert np.array_equal(states[j, :i + 1], rst) and not states[j, i + 1:].any()
        cut = items[len(rows) - 1][0]
        slack = tol * max(abs(cut), scale)
        assert all(s <= cut + slack for s, _ in got), f"layer {i}: a survivor is not among the best"
        chosen = {k for _, k in got}
        assert len(chosen) == len(got), "a survivor appears twice"
        worst = max(s for s, _ in got)
        for s, b, c in items[:len(rows)]:
            assert (b, c) in chosen or s >= worst - slack, f"layer {i}: a better extension was dropped"
        assert (np.diff(vals[rows, i]) >= 0).all(), "survivors are not ordered by score"
        assert (cids[len(rows):] == -1).all() and np.isinf(vals[len(rows):]).all() and not states[len(rows):].any()
        prev = [tuple(int(t) for t in cids[j, :i + 1]) for j in rows]
        vals_prev = [vals[j].copy() for j in rows]


def make_ctx(vf, pipe, sp, model, w, K):
    ctx = vf.vf_create(0)
    vf.vf_set_space(ctx, sp)
    vf.vf_set_pipeline(ctx, np.repeat(pipe[None], K, axis=0))
    vf.vf_set_model(ctx, model, w)

    def run(last):
        vf.vf_reset_state(ctx)
        st, cids, vals, nb = vf.vf_beam_search(ctx, 0, last)
        return cids.cpu().numpy(), vals.cpu().numpy(), st.cpu().numpy(), int(nb.cpu()[0])
    return ctx, run


@pytest.mark.parametrize("K", [1, 4, 16, 40])
def test_beam_fused_bf16(vf, ovf, K):
    sp = I.make_space([1, 2, 3, 8], [1, 2, 5], [1, 4, 16], [(0, 1, 2), (2, 1, 0), (1, 0, 2)], 2, 2,
                      [I.ROOT, I.L1, I.L2, I.INLINE], 2, 256)
    pipe = I.random_pipeline(4, 41)
    dims = [256, 512, 512, 1]
    w = I.mlp_weights(dims, 3, bias_std=0.1)
    model = I.model_record(I.MLP, dims, I.BF16)
    ctx, run = make_ctx(vf, pipe, sp, model, w, K)
    check_beam(ovf, pipe, sp, model, w, run, K, TOL[1])
    cids, vals, st, nb = run(len(pipe) - 1)
    if K == 1:
        vf.vf_reset_state(ctx)
        gs, gc, gv = vf.vf_greedy_schedule(ctx)
        assert np.array_equal(gc.cpu().numpy(), cids) and np.array_equal(gv.cpu().numpy(), vals)
        assert np.array_equal(gs.cpu().numpy(), st)
    vf.vf_destroy(ctx)


@pytest.mark.parametrize("K", [6, 24])
def test_beam_fp32_tiny_config_with_ties(vf, ovf, K):
    """The tiny conv+ReLU config has candidates with identical features, hence exactly
    equal scores: the (score, parent, candidate id) order decides, as in the checker
    (few survivors: rounds of block minima; more: sorted keys)."""
    pipe, sp = I.tiny_conv_relu(), I.tiny_space()
    dims = [64, 128, 128, 1]
    w = I.mlp_weights(dims, 0)
    model = I.model_record(I.MLP, dims, I.FP32)
    ctx, run = make_ctx(vf, pipe, sp, model, w, K)
    check_beam(ovf, pipe, sp, model, w, run, K, TOL[0])
    cids, vals, st, nb = run(1)
    ref = ovf.beam(pipe, sp, K, model, w)
    assert np.array_equal(ref["cids"], cids) and ref["n_beams"] == nb
    vf.vf_destroy(ctx)


def test_beam_general_widths_and_prefix(vf, ovf):
    """A model outside the fused path (features materialised, scores masked afterwards), and a
    search that starts from a committed prefix (the way Algorithm 2 completes schedules)."""
    sp = I.make_space([1, 2, 4], [1, 2], [1, 4], [(0, 1, 2), (2, 1, 0)], 2, 1,
                      [I.ROOT, I.L1, I.L2, I.INLINE], 1, 64)
    pipe = I.random_pipeline(4, 52)
    dims = [64, 96, 32, 1]
    w = I.mlp_weights(dims, 9, bias_std=0.1)
    model = I.model_record(I.MLP, dims, I.BF16)
    ctx, run = make_ctx(vf, pipe, sp, model, w, 5)
    check_beam(ovf, pipe, sp, model, w, run, 5, TOL[1])
    cids, vals, st, nb = run(3)
    ref = ovf.beam(pipe, sp, 5, model, w)
    if np.array_equal(ref["cids"], cids):                    # no decision inside the tolerance
        assert ref["n_beams"] == nb
    # from the best schedule's first decision onwards
    first = int(cids[0, 0])
    vf.vf_set_state(ctx, np.full((5, 1), first, np.int32))
    st2, c2, v2, nb2 = vf.vf_beam_search(ctx, first=1)
    c2 = c2.cpu().numpy()
    assert (c2[c2[:, 0] >= 0, 0] == first).all() and c2[0].tolist() == cids[0].tolist()
    with pytest.raises(vf.VfError):
        vf.vf_beam_search(ctx, first=0)                      # not the next stage
    other = I.random_pipeline(4, 53)
    vf.vf_set_pipeline(ctx, np.stack([pipe, pipe, other, pipe, pipe]))
    with pytest.raises(vf.VfError) as e:
        vf.vf_beam_search(ctx)                               # slots must hold one network
    assert e.value.code == vf.VF_EINVAL
    vf.vf_destroy(ctx)


def test_beam_without_survivors(vf, ovf):
    pipe, sp = I.tiny_conv_relu(), I.tiny_space()
    dims = [64, 32, 1]
    w = I.mlp_weights(dims, 0); w[:] = np.nan
    ctx, run = make_ctx(vf, pipe, sp, I.model_record(I.MLP, dims, I.BF16), w, 3)
    cids, vals, st, nb = run(1)
    assert (cids == -1).all() and np.isinf(vals).all() and not st.any() and nb == 1
    vf.vf_destroy(ctx)
