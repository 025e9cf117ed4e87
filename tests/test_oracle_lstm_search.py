"""Pins for the CPU checker's search guided by the recurrent value network (Sec. 3.2: an
LSTM over the per-stage features of the pipeline, one prediction per timestep, summed):
the sequence form of a state, and Algorithm 1 / beam search / noisy rollouts on top of it."""
import numpy as np
import pytest
import torch

from paper_2011_14486_amd import inputs as I
from tests.test_oracle_score import torch_lstm


def small_problem(seed, S=4, F=64):
    sp = I.make_space([1, 4], [1, 2], [1, 2], [(0, 1, 2), (2, 1, 0)], 2, 1,
                      [I.ROOT, I.L1, I.L2, I.INLINE], 1, F)
    return I.random_pipeline(S, seed, max_hw=9, max_c=6), sp


def bf16_bits(v):
    """Library conversion float32 -> bf16 bit patterns."""
    t = torch.from_numpy(np.ascontiguousarray(v, np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def any_schedule(ovf, pipe, sp, pick):
    """A valid complete schedule: at every stage the pick-th valid candidate (modulo)."""
    cids = []
    for i in range(len(pipe)):
        _, valid, _ = ovf.enumerate_candidates(pipe, sp, cids, i)
        ids = np.flatnonzero(valid)
        cids.append(int(ids[pick % len(ids)]))
    return cids


@pytest.mark.parametrize("seed,F", [(0, 64), (1, 256), (2, 64), (5, 256)])
def test_sequence_form_is_composed_from_the_feature_columns(ovf, seed, F):
    """Timestep t of a candidate state is: the column that stage t's committed candidate had
    when it was decided (t < i), the candidate's own column (t = i), the intrinsic block of
    stage t and zeros (t > i); normalised, bf16.  Composed here from ovf.featurize."""
    pipe, sp = small_problem(seed, S=5, F=F)
    S, M = len(pipe), I.space_dense_count(sp)
    sched = any_schedule(ovf, pipe, sp, 3)
    other = any_schedule(ovf, pipe, sp, 0)
    cols = [ovf.featurize(pipe, sp, sched[:t], t)[:64] for t in range(S)]
    for t in range(S):
        # the intrinsic block does not depend on the schedule, nor on the candidate
        alt = ovf.featurize(pipe, sp, other[:t], t)[:16]
        assert np.array_equal(alt[:, 0], cols[t][:16, 0]) and (cols[t][:16, :M] == cols[t][:16, :1]).all()
    for i in (0, 2, S - 1):
        x, valid = ovf.sequences(pipe, sp, sched[:i], i)
        assert x.shape == (M, S, 64)
        assert np.array_equal(valid, cols[i][16, :M].astype(np.uint8))
        want = np.zeros((M, S, 64), np.int32)
        for t in range(S):
            if t < i:
                want[:, t, :] = cols[t][:, sched[t]]
            elif t == i:
                want[:, t, :] = cols[i][:, :M].T
            else:
                want[:, t, :16] = cols[t][:16, 0]
        assert np.array_equal(x, bf16_bits(ovf.plog2(want)))
        assert (want[valid == 0][:, i, 16:] == 0).all()


def lstm_scan(ovf, pipe, sp, F, H, w, bf16):
    """Algorithm 1 re-done here: sequences from the checker, the network from torch."""
    cids, vals = [], []
    for i in range(len(pipe)):
        x, valid = ovf.sequences(pipe, sp, cids, i)
        xs = (x.astype(np.uint32) << 16).view(np.float32)
        v = torch_lstm(F, H, w, xs, bf16).astype(np.float32)
        best, arg = np.inf, -1
        for cid in range(len(v)):
            if valid[cid] and v[cid] < best:
                best, arg = v[cid], cid
        cids.append(arg); vals.append(best)
    return np.array(cids), np.array(vals)


@pytest.mark.parametrize("seed,dtype", [(0, I.FP32), (1, I.FP32), (2, I.BF16), (3, I.BF16)])
def test_greedy_with_the_recurrent_network_against_library_lstm(ovf, seed, dtype):
    pipe, sp = small_problem(seed)
    H = 12
    w = I.lstm_weights(64, H, seed=seed, bias_std=0.2)
    m = I.model_record(I.LSTM, [64, H, 1], dtype)
    g = ovf.greedy(pipe, sp, m, w)
    cids, vals = lstm_scan(ovf, pipe, sp, 64, H, w, dtype == I.BF16)
    assert np.array_equal(g["cids"], cids)
    assert np.max(np.abs(g["values"] - vals) / np.maximum(np.abs(vals), 1.0)) < 2e-6
    # each valid candidate costs one evaluation of V
    n = 0
    for i in range(len(pipe)):
        n += int(ovf.enumerate_candidates(pipe, sp, list(cids[:i]), i)[2])
    assert g["n_evals"] == n


def test_constant_network_closed_form(ovf):
    """Zero matrices: every timestep's hidden state is the same closed form of the biases,
    so V = S * (w . h + b) for every state and the scan keeps the first valid candidate."""
    pipe, sp = small_problem(4, S=5)
    H, S = 8, 5
    rng = np.random.default_rng(0)
    bih, bhh = rng.standard_normal(4 * H) * 0.5, rng.standard_normal(4 * H) * 0.5
    wh, bh = rng.standard_normal(H), 0.3
    w = np.concatenate([np.zeros(4 * H * 64), np.zeros(4 * H * H), bih, bhh, wh, [bh]]).astype(np.float32)
    g = ovf.greedy(pipe, sp, I.model_record(I.LSTM, [64, H, 1], I.FP32), w)
    z = bih.astype(np.float32).astype(np.float64) + bhh.astype(np.float32).astype(np.float64)
    sig = lambda a: 1 / (1 + np.exp(-a))
    i_, f_, g_, o_ = sig(z[:H]), sig(z[H:2 * H]), np.tanh(z[2 * H:3 * H]), sig(z[3 * H:])
    c, v = np.zeros(H), 0.0
    for _ in range(S):
        c = f_ * c + i_ * g_
        v += float(wh.astype(np.float32).astype(np.float64) @ (o_ * np.tanh(c))) + np.float32(bh)
    assert np.allclose(g["values"], v, rtol=1e-6)
    first_valid = any_schedule(ovf, pipe, sp, 0)
    assert g["cids"].tolist() == first_valid


def test_unscheduled_stages_and_the_prefix_reach_the_prediction(ovf):
    """The value of a state depends on the committed prefix and on the stages still to come:
    changing a later stage's shape, or an earlier decision, changes V of the same candidate."""
    pipe, sp = small_problem(0, S=4)
    H = 12
    w = I.lstm_weights(64, H, seed=1, bias_std=0.2)
    m = I.model_record(I.LSTM, [64, H, 1], I.FP32)
    sched = any_schedule(ovf, pipe, sp, 1)
    x, valid = ovf.sequences(pipe, sp, sched[:1], 1)
    cid = int(np.flatnonzero(valid)[0])
    v0 = ovf.score_lstm(m, w, x[cid:cid + 1])[0]
    later = pipe.copy(); later[3, 12] = 2   # element size of the last stage: its intrinsic block only
    x2, _ = ovf.sequences(later, sp, sched[:1], 1)
    assert np.array_equal(x2[cid, :3], x[cid, :3]) and not np.array_equal(x2[cid, 3], x[cid, 3])
    assert ovf.score_lstm(m, w, x2[cid:cid + 1])[0] != v0
    other0 = any_schedule(ovf, pipe, sp, 2)[0]
    assert other0 != sched[0]
    x3, valid3 = ovf.sequences(pipe, sp, [other0], 1)
    assert not np.array_equal(x3[cid, 0], x[cid, 0])


@pytest.mark.parametrize("seed", range(3))
def test_beam_width_one_and_noise_free_rollout_are_the_greedy_scan(ovf, seed):
    pipe, sp = small_problem(seed + 10)
    H = 8
    w = I.lstm_weights(64, H, seed=seed, bias_std=0.1)
    m = I.model_record(I.LSTM, [64, H, 1], I.BF16)
    g = ovf.greedy(pipe, sp, m, w)
    b = ovf.beam(pipe, sp, 1, m, w)
    assert np.array_equal(b["cids"][0], g["cids"]) and np.array_equal(b["values"][0], g["values"])
    r = ovf.rollouts(pipe, sp, m, w, 0.0, 5, 2)
    assert np.array_equal(r["cids"][1], g["cids"]) and np.array_equal(r["values"][0], g["values"])
    wide = ovf.beam(pipe, sp, 4, m, w)
    assert wide["values"][0][-1] <= g["values"][-1]


def test_model_shape_is_checked(ovf):
    pipe, sp = small_problem(0)
    w = I.lstm_weights(32, 8, seed=0)
    with pytest.raises(ovf.OracleError):
        ovf.greedy(pipe, sp, I.model_record(I.LSTM, [32, 8, 1], I.FP32), w)


def test_beam_rows_carry_the_value_of_their_own_prefix(ovf):
    """Every surviving row's value at layer i is V of that row's own first i+1 decisions
    (recomputed from the sequence form), and an exhaustive width finds the brute-force best
    complete schedule."""
    sp = I.make_space([1, 2], [1], [1, 2], [(0, 1, 2)], 1, 1, [I.ROOT, I.L1], 1, 64)
    pipe = I.random_pipeline(3, 21, max_hw=6, max_c=4)
    H, S = 8, 3
    w = I.lstm_weights(64, H, seed=4, bias_std=0.3)
    m = I.model_record(I.LSTM, [64, H, 1], I.FP32)

    def value_of(cids):
        x, valid = ovf.sequences(pipe, sp, cids[:-1], len(cids) - 1)
        assert valid[cids[-1]]
        return ovf.score_lstm(m, w, x[cids[-1]:cids[-1] + 1])[0]

    b = ovf.beam(pipe, sp, 3, m, w)
    assert b["n_beams"] >= 2
    for j in range(b["n_beams"]):
        row = [int(c) for c in b["cids"][j]]
        for i in range(S):
            assert b["values"][j][i] == value_of(row[:i + 1])
    assert len({tuple(r) for r in b["cids"][:b["n_beams"]].tolist()}) == b["n_beams"]
    # exhaustive
    complete = [[]]
    for i in range(S):
        nxt = []
        for pre in complete:
            _, valid, _ = ovf.enumerate_candidates(pipe, sp, pre, i)
            nxt += [pre + [int(c)] for c in np.flatnonzero(valid)]
        complete = nxt
    best = min(value_of(c) for c in complete)
    wide = ovf.beam(pipe, sp, len(complete) + 5, m, w)
    assert wide["n_beams"] == len(complete) and wide["values"][0][-1] == best
