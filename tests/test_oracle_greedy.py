"""Pins for the CPU checker's Algorithm 1 loop."""
import itertools

import numpy as np
import pytest

from paper_2011_14486_amd import inputs as I

NCORES = 18


def stage_cost(core):
    """An additive integer cost of one committed stage, from its core features:
    compute time with vector lanes and cores, plus bytes moved."""
    lanes, tasks = max(int(core[27]), 1), max(int(core[30]), 1)
    return (int(core[40]) * 16) // (lanes * min(tasks, NCORES)) + int(core[51]) + int(core[50])


def tiny_problem(seed):
    rng = np.random.default_rng(seed)
    sp = I.make_space([1, 4], [1], [1, 2], [(0, 1, 2), (2, 1, 0)], 2, 1,
                      [I.ROOT, I.L1, I.L2, I.INLINE], 1, 64)
    k = int(rng.choice([1, 3]))
    pipe = np.array([
        I.stage_record(I.POINTWISE, 8, 8, 4, anchor=-1, n_consumers=0, in0=1),
        I.stage_record(I.CONV, 8, 8, 4, RC=int(rng.integers(1, 5)), KH=k, KW=k, anchor=0, in0=2),
        I.stage_record(I.POINTWISE, 8 + k - 1, 8 + k - 1, 4, anchor=1),
    ], np.int32)
    return pipe, sp


class ExactV:
    """V*(s): cost of the committed stages plus the minimum over all completions,
    by exhaustive recursion (Sec. 2: the true value function)."""

    def __init__(self, ovf, pipe, sp):
        self.ovf, self.pipe, self.sp = ovf, pipe, sp
        self.S = len(pipe)
        self.memo = {}
        self.leaves = 0

    def candidates(self, prefix):
        feat = self.ovf.featurize(self.pipe, self.sp, list(prefix), len(prefix))
        ok = np.flatnonzero(feat[16] == 1)
        return [(int(c), stage_cost(feat[:64, c])) for c in ok]

    def completion(self, prefix):
        """min cost of the stages not in prefix"""
        if len(prefix) == self.S:
            self.leaves += 1
            return 0
        if prefix not in self.memo:
            self.memo[prefix] = min(cost + self.completion(prefix + (c,))
                                    for c, cost in self.candidates(prefix))
        return self.memo[prefix]

    def prefix_cost(self, prefix):
        _, cf = self.ovf.states(self.pipe, self.sp, list(prefix))
        return sum(stage_cost(cf[j]) for j in range(len(prefix)))


@pytest.mark.parametrize("seed", range(3))
def test_greedy_with_exact_value_function_is_optimal(ovf, seed):
    """Sec. 2: with the true value function the greedy scan finds the optimum.  The
    optimum is found independently by brute force over every complete schedule."""
    pipe, sp = tiny_problem(seed)
    ex = ExactV(ovf, pipe, sp)
    best = ex.completion(())
    # brute force over the full product space, written without the recursion's memo
    brute = None
    n_complete = 0
    for c0, k0 in ex.candidates(()):
        for c1, k1 in ex.candidates((c0,)):
            for c2, k2 in ex.candidates((c0, c1)):
                n_complete += 1
                tot = k0 + k1 + k2
                brute = tot if brute is None else min(brute, tot)
    assert 1000 < n_complete <= 2 * 10 ** 5 and brute == best

    chosen = []
    evals = 0
    for i in range(3):
        pre = tuple(chosen)
        base = ex.prefix_cost(pre)
        table = {c: base + k + ex.completion(pre + (c,)) for c, k in ex.candidates(pre)}

        def vstar(user, stage, cid, core, table=table, i=i):
            assert stage == i and core[16] == 1
            return float(table[cid])
        g = ovf.greedy(pipe, sp, vfun=vstar, first=i, last=i, prefix_cids=chosen)
        c = int(g["cids"][i])
        assert g["n_evals"] == len(table)
        evals += g["n_evals"]
        assert float(g["values"][i]) == best                 # V* of the kept state is the optimum
        assert c == min(k for k, v in table.items() if v == best)   # first minimum on ties
        chosen.append(c)
    assert ex.prefix_cost(tuple(chosen)) == brute
    # N*M evaluations instead of M^N complete schedules
    assert evals < n_complete


def test_greedy_counts_and_prefix_carry(ovf):
    pipe, sp = tiny_problem(5)
    dims = [64, 16, 1]
    w = I.mlp_weights(dims, seed=1, bias_std=0.1)
    mod = I.model_record(I.MLP, dims, I.FP32)
    full = ovf.greedy(pipe, sp, mod, w)
    # stage by stage through the public pieces: featurize -> score -> argmin
    pre, nval = [], 0
    for i in range(3):
        feat = ovf.featurize(pipe, sp, pre, i)
        dec, valid, nv = ovf.enumerate_candidates(pipe, sp, pre, i)
        sc = ovf.score_mlp(mod, w, feat, M=ovf.dense_count(sp))
        bi, bv = ovf.argmin(sc, valid=valid)
        assert bi[0] == full["cids"][i] and bv[0] == full["values"][i]
        srt = np.sort(sc[valid[:len(sc)] == 1])
        assert full["top2"][i] == srt[1]
        pre.append(int(bi[0])); nval += nv
    assert full["n_evals"] == nval                          # sum_i M_i value-function evaluations
    st, _ = ovf.states(pipe, sp, pre)
    assert np.array_equal(st, full["states"])
    # resuming from a prefix gives the same tail
    tail = ovf.greedy(pipe, sp, mod, w, first=1, prefix_cids=pre[:1])
    assert np.array_equal(tail["cids"], full["cids"]) and np.array_equal(tail["values"][1:], full["values"][1:])
    # forcing another valid candidate at stage 0 changes what follows consistently
    _, v0, _ = ovf.enumerate_candidates(pipe, sp, [], 0)
    other = int(np.flatnonzero(v0)[-1])
    forced = ovf.greedy(pipe, sp, mod, w, forced=[other, -1, -1])
    again = ovf.greedy(pipe, sp, mod, w, first=1, prefix_cids=[other])
    assert forced["cids"][0] == other and np.array_equal(forced["cids"][1:], again["cids"][1:])


def test_greedy_without_a_winner(ovf):
    """v_i stays at +infinity when no candidate is smaller: the stage gets no state and
    the schedule ends there."""
    pipe, sp = tiny_problem(1)
    dims = [64, 8, 1]
    w = I.mlp_weights(dims, seed=1)
    w[:] = np.nan
    g = ovf.greedy(pipe, sp, I.model_record(I.MLP, dims, I.FP32), w)
    assert g["cids"].tolist() == [-1, -1, -1] and np.isinf(g["values"]).all()
    # a space in which nothing is valid: every factor exceeds the extents
    sp2 = I.make_space([32], [32], [32], [(0, 1, 2)], 1, 1, [I.ROOT], 1, 64)
    w = I.mlp_weights(dims, seed=1)
    g = ovf.greedy(pipe, sp2, I.model_record(I.MLP, dims, I.FP32), w)
    assert g["cids"].tolist() == [-1, -1, -1] and g["n_evals"] == 0


def test_greedy_on_the_tiny_config(ovf):
    pipe, sp = I.tiny_conv_relu(), I.tiny_space()
    dims = [64, 128, 128, 1]
    g = ovf.greedy(pipe, sp, I.model_record(I.MLP, dims, I.FP32), I.mlp_weights(dims, 0))
    assert g["n_evals"] == 4800 and (g["cids"] >= 0).all()
    assert (g["values"] <= g["top2"]).all()
