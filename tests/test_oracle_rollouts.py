"""Pins for the CPU checker's noisy greedy rollouts (Sec. 3.1 / Algorithm 2:
BestSchedule(n, V_eps) adds a small random noise to the predictions)."""
import os

import numpy as np
import pytest

from paper_2011_14486_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers(ovf):
    n = 0
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        w = [int(t, 16) for t in line]
        assert ovf.philox4x32_10(w[0:4], w[4:6]).tolist() == w[6:10]
        n += 1
    assert n == 3


def test_noise_is_the_first_word_scaled(ovf):
    seed = 0x0123456789abcdef
    for r, s, c in [(0, 0, 0), (3, 7, 4095), (99, 19, 123456), (1, 0, 2 ** 30)]:
        x = int(ovf.philox4x32_10([c, s, r, 0], [seed & 0xffffffff, seed >> 32])[0])
        assert ovf.noise(seed, r, s, c) == (x >> 8) / 2.0 ** 23 - 1.0
    v = np.array([ovf.noise(5, 1, 2, c) for c in range(20000)])
    assert -1.0 <= v.min() and v.max() < 1.0 and abs(v.mean()) < 0.02 and abs(v.var() - 1 / 3) < 0.01
    assert ovf.noise(5, 1, 2, 7) != ovf.noise(5, 2, 2, 7) != ovf.noise(5, 1, 3, 7) != ovf.noise(6, 1, 2, 7)


def problem(seed=3):
    sp = I.make_space([1, 2, 4], [1, 2], [1, 4], [(0, 1, 2), (2, 1, 0)], 2, 1,
                      [I.ROOT, I.L1, I.L2, I.INLINE], 1, 64)
    pipe = I.random_pipeline(3, seed, max_hw=12, max_c=8)
    dims = [64, 16, 1]
    return pipe, sp, I.model_record(I.MLP, dims, I.FP32), I.mlp_weights(dims, seed, bias_std=0.1)


def test_zero_noise_is_the_greedy_scan(ovf):
    pipe, sp, m, w = problem()
    g = ovf.greedy(pipe, sp, m, w)
    r = ovf.rollouts(pipe, sp, m, w, 0.0, 7, 3)
    for k in range(3):
        assert np.array_equal(r["cids"][k], g["cids"]) and np.array_equal(r["values"][k], g["values"])


def test_rollout_is_the_scan_over_noisy_scores(ovf):
    """Each rollout's decision is the first minimum of score + eps*noise, computed here from
    the checker's plain scores and its noise primitive; the kept value is the noisy one."""
    pipe, sp, m, w = problem(4)
    eps, seed = np.float32(0.25), 42
    M = ovf.dense_count(sp)
    r = ovf.rollouts(pipe, sp, m, w, float(eps), seed, 5, first_rollout=10)
    plain = ovf.greedy(pipe, sp, m, w)
    assert any(not np.array_equal(r["cids"][k], plain["cids"]) for k in range(5))   # the noise matters
    assert len({tuple(r["cids"][k]) for k in range(5)}) > 1                          # rollouts differ
    for k in range(5):
        pre = []
        for i in range(len(pipe)):
            feat = ovf.featurize(pipe, sp, pre, i)
            sc = ovf.score_mlp(m, w, feat, M=M)
            nz = np.array([ovf.noise(seed, 10 + k, i, c) for c in range(M)], np.float32)
            noisy = (sc + (eps * nz).astype(np.float32)).astype(np.float32)
            noisy[feat[16, :M] == 0] = np.inf
            best = int(np.argmin(noisy))
            assert r["cids"][k, i] == best and r["values"][k, i] == noisy[best]
            assert r["top2"][k, i] == np.sort(noisy)[1]
            pre.append(best)
    again = ovf.rollouts(pipe, sp, m, w, float(eps), seed, 5, first_rollout=10)
    assert np.array_equal(again["cids"], r["cids"]) and np.array_equal(again["values"], r["values"])
    shifted = ovf.rollouts(pipe, sp, m, w, float(eps), seed, 2, first_rollout=12)
    assert np.array_equal(shifted["cids"], r["cids"][2:4])                           # rollout ids, not positions


def test_decision_scores_are_what_the_scan_sees(ovf):
    """ovf.decision_scores exposes the per-decision scores of the greedy scan / the rollouts:
    plain, they are score_mlp over featurize with the validity row; noisy, the first minimum and
    the runner-up over the valid ones are what ovf.rollouts reports, layer by layer."""
    pipe, sp, m, w = problem(4)
    M = ovf.dense_count(sp)
    g = ovf.greedy(pipe, sp, m, w)
    for i in range(len(pipe)):
        sc, ok = ovf.decision_scores(pipe, sp, m, w, g["cids"][:i], i)
        feat = ovf.featurize(pipe, sp, g["cids"][:i], i)
        assert np.array_equal(ok, feat[16, :M] == 1)
        assert np.array_equal(sc[ok], ovf.score_mlp(m, w, feat, M=M)[ok])
        best = int(np.flatnonzero(ok)[np.argmin(sc[ok])])
        assert best == g["cids"][i] and sc[best] == g["values"][i]
    eps, seed = 0.25, 42
    r = ovf.rollouts(pipe, sp, m, w, eps, seed, 3, first_rollout=10)
    for k in range(3):
        for i in range(len(pipe)):
            sc, ok = ovf.decision_scores(pipe, sp, m, w, r["cids"][k, :i], i, eps, seed, 10 + k)
            s = np.where(ok, sc, np.inf)
            assert int(np.argmin(s)) == r["cids"][k, i] and s.min() == r["values"][k, i]
            assert np.sort(s)[1] == r["top2"][k, i]
    with pytest.raises(ovf.OracleError):
        ovf.decision_scores(pipe, sp, m, w, [0] * 5, 5)        # no such stage
