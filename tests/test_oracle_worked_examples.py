"""Pins the CPU checker's enumeration and features to hand-derived worked examples
(tests/golden/*.txt) and to closed-form candidate counts."""
import os

import numpy as np

from paper_2011_14486_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def load(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].strip()
        if not line:
            continue
        k, v = [t.strip() for t in line.split("=")]
        out[k] = int(v, 0)
    return out


def check(ovf, pipe, space, gold):
    pre = [gold["prefix_cid_0"]]
    dec, valid, nv = ovf.enumerate_candidates(pipe, space, pre, 1)
    feat = ovf.featurize(pipe, space, pre, 1)
    cid = gold["cid"]
    assert valid[cid] == gold["valid"]
    if "dec_packed" in gold:
        assert int(dec[cid]) == gold["dec_packed"]
    if "n_valid" in gold:
        assert nv == gold["n_valid"] == int(valid.sum())
    for k, v in gold.items():
        if k.startswith("f") and k[1:].isdigit():
            assert int(feat[int(k[1:]), cid]) == v, (k, int(feat[int(k[1:]), cid]), v)
    return feat, valid


def test_example_a_conv_in_relu_tile(ovf):
    pipe = np.array([I.stage_record(I.POINTWISE, 16, 16, 8, anchor=-1, n_consumers=0, in0=1),
                     I.stage_record(I.CONV, 16, 16, 8, RC=8, KH=3, KW=3, anchor=0)], np.int32)
    space = I.make_space([1, 4], [1, 8], [1, 2], [(0, 1, 2), (1, 2, 0)], 2, 2,
                         [I.ROOT, I.L1, I.L2, I.INLINE], 2, 64)
    assert ovf.dense_count(space) == 512
    gold = load("worked_conv_in_relu_tile.txt")
    assert len([k for k in gold if k.startswith("f")]) == 64  # the whole core vector
    check(ovf, pipe, space, gold)


def test_example_b_halo_under_strided_depthwise(ovf):
    pipe = np.array([I.stage_record(I.DWCONV, 8, 8, 6, RC=1, KH=3, KW=3, stride=2, anchor=-1, n_consumers=0, in0=1),
                     I.stage_record(I.POINTWISE, 17, 17, 6, anchor=0)], np.int32)
    space = I.make_space([1, 2, 4], [1, 2], [1, 3], [(0, 1, 2), (2, 0, 1)], 2, 2,
                         [I.ROOT, I.L1, I.L2, I.INLINE], 1, 64)
    assert ovf.dense_count(space) == 384
    gold = load("worked_pointwise_under_strided_dw.txt")
    feat, valid = check(ovf, pipe, space, gold)
    c = gold["l2_cid"]
    assert valid[c] == 1
    for k, v in gold.items():
        if k.startswith("l2_f"):
            assert int(feat[int(k[4:]), c]) == v, k


def test_example_c_inline_into_conv(ovf):
    pipe = np.array([I.stage_record(I.CONV, 8, 8, 8, RC=4, KH=3, KW=3, anchor=-1, n_consumers=0, in0=1),
                     I.stage_record(I.POINTWISE, 10, 10, 4, anchor=0)], np.int32)
    space = I.make_space([1, 4], [1, 2], [1], [(0, 1, 2)], 2, 1, [I.ROOT, I.INLINE], 1, 64)
    assert ovf.dense_count(space) == 16
    check(ovf, pipe, space, load("worked_inline_into_conv.txt"))


def test_tiny_config_counts(ovf):
    """Closed form: factors {1,2,4,8,16}^3 x 6 orders x vec x par x {ROOT, INLINE}: M = 6000.
    8-channel 16x16 conv: f_c = 16 > 8 is no split and a conv cannot be inlined:
    5*5*4*6*2*2 = 2400.  The ReLU listed first has no anchor: ROOT only, 2400.  Listed
    second with the conv as anchor it gains the single canonical INLINE candidate: 2401."""
    sp = I.tiny_space()
    assert ovf.dense_count(sp) == 6000 and ovf.padded_count(sp) == 6144
    p = I.tiny_conv_relu()
    _, v0, n0 = ovf.enumerate_candidates(p, sp, [], 0)
    assert n0 == 2400
    c0 = int(np.flatnonzero(v0)[7])
    _, v1, n1 = ovf.enumerate_candidates(p, sp, [c0], 1)
    assert n1 == 2400
    q = I.tiny_conv_relu("input_first")
    _, w0, m0 = ovf.enumerate_candidates(q, sp, [], 0)
    assert m0 == 2400
    _, w1, m1 = ovf.enumerate_candidates(q, sp, [int(np.flatnonzero(w0)[0])], 1)
    assert m1 == 2401
    assert w1[3000] == 1 and w1[3001:].sum() == 0  # the canonical inline id is icat=1, rest 0


def test_workload_shapes():
    """The synthetic pipelines have the documented sizes (bookkeeping only)."""
    r = I.resnet18_shaped()
    m = I.mobilenetv2_shaped()
    assert r.shape == (20, 16) and m.shape == (100, 16)
    assert I.space_dense_count(I.resnet18_space()) == 4096
    assert I.space_dense_count(I.mobilenetv2_space()) == 16384

    def macs(p):
        return sum(int(w[1]) * w[2] * w[3] * (int(w[4]) * w[5] * w[6] if w[0] in (0, 1) else 1) for w in p)
    assert macs(r) == 784301056 and macs(m) == 427145152
    assert max(int(w[1]) * w[2] * w[3] * w[4] * w[5] * w[6] for w in r) == 115605504
    for p in (r, m):
        for j, w in enumerate(p):
            assert -1 <= w[8] < j
    # a stage whose output feeds two consumers (the residual split) is ROOT-only
    assert sorted(set(r[:, 9].tolist())) == [0, 1, 2]
