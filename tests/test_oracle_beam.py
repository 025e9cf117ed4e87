"""Pins for the CPU checker's beam search (the V-guided search the paper runs next to
the greedy scan, Secs. 3.1 and 4.1)."""
import numpy as np
import pytest

from paper_2011_14486_amd import inputs as I


def small_problem(seed, S=3):
    sp = I.make_space([1, 4], [1], [1, 2], [(0, 1, 2), (2, 1, 0)], 2, 1,
                      [I.ROOT, I.L1, I.L2, I.INLINE], 1, 64)
    return I.random_pipeline(S, seed, max_hw=9, max_c=6), sp


@pytest.mark.parametrize("seed", range(4))
def test_width_one_is_the_greedy_scan(ovf, seed):
    pipe, sp = small_problem(seed)
    dims = [64, 16, 1]
    w = I.mlp_weights(dims, seed, bias_std=0.1)
    m = I.model_record(I.MLP, dims, I.FP32)
    g = ovf.greedy(pipe, sp, m, w)
    b = ovf.beam(pipe, sp, 1, m, w)
    assert np.array_equal(b["cids"][0], g["cids"]) and np.array_equal(b["values"][0], g["values"])
    assert b["n_evals"] == g["n_evals"] and b["n_beams"] == 1


def test_beam_recovers_what_greedy_misses(ovf):
    """A value function that makes the locally best first decision a dead end: candidate
    0 scores 1.0 and candidate 1 scores 1.1 at the first layer; at the second layer every
    state below candidate 0 scores 5, below candidate 1 the first candidate scores 0."""
    sp = I.make_space([1, 2], [1], [1], [(0, 1, 2)], 1, 1, [I.ROOT], 1, 64)
    pipe = np.array([I.stage_record(I.POINTWISE, 4, 4, 4, anchor=-1, n_consumers=0, in0=1),
                     I.stage_record(I.POINTWISE, 4, 4, 4, anchor=0)], np.int32)
    # both candidates of both stages are valid (f = 1 or 2 on a 4-wide loop)
    _, cf = ovf.states(pipe, sp, [1])
    below_one = int(cf[0, 54])  # n_tiles of candidate 1 at stage 0, seen at stage 1 as row 57

    def v(user, stage, cid, core):
        if stage == 0:
            return 1.0 + 0.1 * cid
        return (0.0 if cid == 0 else 0.5) if core[57] == below_one else 5.0 + cid

    g = ovf.greedy(pipe, sp, vfun=v)
    assert g["cids"].tolist() == [0, 0] and g["values"].tolist() == [1.0, 5.0]
    b = ovf.beam(pipe, sp, 2, vfun=v)
    assert b["cids"].tolist() == [[1, 0], [1, 1]]
    assert b["values"].tolist() == [[np.float32(1.1), 0.0], [np.float32(1.1), 0.5]]
    assert b["n_beams"] == 2 and b["n_evals"] == 2 + 4
    b3 = ovf.beam(pipe, sp, 3, vfun=v)       # only two states exist after the first layer
    assert b3["cids"].tolist() == [[1, 0], [1, 1], [0, 0]] and b3["n_beams"] == 3
    b8 = ovf.beam(pipe, sp, 8, vfun=v)       # all four complete schedules, then unused rows
    assert b8["cids"][:4].tolist() == [[1, 0], [1, 1], [0, 0], [0, 1]] and b8["n_beams"] == 4
    assert (b8["cids"][4:] == -1).all() and np.isinf(b8["values"][4:]).all()


def test_ties_keep_parent_then_candidate_order(ovf):
    sp = I.make_space([1, 2, 4], [1], [1], [(0, 1, 2)], 1, 1, [I.ROOT], 1, 64)
    pipe = np.array([I.stage_record(I.POINTWISE, 4, 4, 4, anchor=-1, n_consumers=0, in0=1),
                     I.stage_record(I.POINTWISE, 4, 4, 4, anchor=0)], np.int32)
    b = ovf.beam(pipe, sp, 4, vfun=lambda u, s, c, core: 7.0)
    assert b["cids"].tolist() == [[0, 0], [0, 1], [0, 2], [1, 0]]
    nan = ovf.beam(pipe, sp, 4, vfun=lambda u, s, c, core: float("nan"))
    assert (nan["cids"] == -1).all() and np.isinf(nan["values"]).all()
    # a dead end after the first layer keeps the schedules found so far, without a second entry
    dead = ovf.beam(pipe, sp, 2, vfun=lambda u, s, c, core: float(c) if s == 0 else float("inf"))
    assert dead["cids"].tolist() == [[0, -1], [1, -1]] and dead["values"][:, 0].tolist() == [0.0, 1.0]


@pytest.mark.parametrize("seed", range(3))
def test_wide_beam_is_exhaustive(ovf, seed):
    """With a beam at least as wide as the number of partial schedules nothing is ever cut,
    so the best row is the minimum of V over every complete schedule (brute force)."""
    pipe, sp = small_problem(20 + seed, S=2)
    dims = [64, 8, 1]
    w = I.mlp_weights(dims, seed, bias_std=0.2)
    m = I.model_record(I.MLP, dims, I.FP32)
    M = ovf.dense_count(sp)
    finals = []
    _, v0, _ = ovf.enumerate_candidates(pipe, sp, [], 0)
    for c0 in np.flatnonzero(v0):
        feat = ovf.featurize(pipe, sp, [int(c0)], 1)
        sc = ovf.score_mlp(m, w, feat, M=M)
        for c1 in np.flatnonzero(feat[16, :M]):
            finals.append((float(sc[c1]), int(c0), int(c1)))
    finals.sort()
    b = ovf.beam(pipe, sp, len(finals) + 5, m, w)
    assert b["n_beams"] == len(finals)
    got = [(float(b["values"][j, 1]), int(b["cids"][j, 0]), int(b["cids"][j, 1])) for j in range(len(finals))]
    assert [g[0] for g in got] == [f[0] for f in finals]
    assert sorted(got) == finals
    # and a narrow beam never beats it
    for k in (1, 2, 5):
        assert ovf.beam(pipe, sp, k, m, w)["values"][0, 1] >= finals[0][0]
