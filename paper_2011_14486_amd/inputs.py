"""Seeded synthetic inputs: pipelines, search spaces, value-network weights, raw
feature matrices and feature sequences.

This module only *describes* workloads (shapes, integer records, random numbers).
It holds none of the scheduler's arithmetic: no candidate decoding, no features,
no normalisation, no network evaluation.  Both the HIP library's tests and the CPU
checker's tests draw their inputs from here so that they see identical data.

The paper evaluates on twelve unnamed text / speech / image models (Sec. 4.2) and
never lists them; the pipelines below are synthetic stand-ins with the layer shapes
of well-known image networks.  Pipelines are listed in *scheduling order*, which is
output-first: L_1 is the last layer of the network, so that the layer a stage may be
computed inside (its anchor, a consumer) is always scheduled before it (Sec. 2:
the options for L_{i+1} depend on the loop structure of the layers already
scheduled).
"""
from __future__ import annotations

import numpy as np

# stage kinds
CONV, DWCONV, POINTWISE, ADD = 0, 1, 2, 3
# compute_at levels
ROOT, L1, L2, INLINE = 0, 1, 2, 3

STAGE_WORDS = 16
STATE_WORDS = 16
SPACE_WORDS = 65
MODEL_WORDS = 11

MLP, LSTM = 0, 1
FP32, BF16 = 0, 1

ALL_PERMS = [(0, 1, 2), (0, 2, 1), (1, 0, 2), (1, 2, 0), (2, 0, 1), (2, 1, 0)]
# loop orders (outer -> inner) whose innermost loop is x (dim 0) or c (dim 2)
XC_INNER_PERMS = [(1, 2, 0), (2, 1, 0), (0, 1, 2), (1, 0, 2)]


def stage_record(kind, W, H, C, RC=1, KH=1, KW=1, stride=1, anchor=-1,
                 n_consumers=1, in0=-1, in1=-1, elem_bytes=4):
    """One 16-word stage record: kind, output extents W,H,C, reduced channels RC,
    kernel KH,KW, stride, anchor, n_consumers, producers in0,in1, elem_bytes, 0,0,0."""
    return [kind, W, H, C, RC, KH, KW, stride, anchor, n_consumers, in0, in1,
            elem_bytes, 0, 0, 0]


def make_space(fx, fy, fc, perms, nvec, npar, cats, nsat, F,
               vlen=16, ncores=18, l1_bytes=32 * 1024, l2_bytes=1 << 20):
    """Flat int32 search-space descriptor (65 words):
    nf[3], fac[3][8], nperm, perm[8][3], nvec, npar, ncat, cat[4], nsat,
    vlen, ncores, l1_bytes, l2_bytes, F.
    The machine constants echo the 18-core AVX-512 CPU of the paper's Sec. 4; they
    are model constants, not measurements."""
    w = np.zeros(SPACE_WORDS, dtype=np.int32)
    facs = [list(fx), list(fy), list(fc)]
    for d in range(3):
        assert 1 <= len(facs[d]) <= 8
        w[d] = len(facs[d])
        w[3 + 8 * d: 3 + 8 * d + len(facs[d])] = facs[d]
    assert 1 <= len(perms) <= 8
    w[27] = len(perms)
    for p, perm in enumerate(perms):
        assert sorted(perm) == [0, 1, 2]
        w[28 + 3 * p: 31 + 3 * p] = perm
    w[52] = nvec
    w[53] = npar
    w[54] = len(cats)
    w[55:55 + len(cats)] = cats
    w[59] = nsat
    w[60:65] = [vlen, ncores, l1_bytes, l2_bytes, F]
    return w


def space_dense_count(space):
    """Product of the eight radices (plain bookkeeping, used for buffer sizes)."""
    s = np.asarray(space, dtype=np.int64)
    return int(s[0] * s[1] * s[2] * s[27] * s[52] * s[53] * s[54] * s[59])


def padded(M, to=256):
    return (int(M) + to - 1) // to * to


def model_record(kind, dims, dtype):
    """Flat int32 model descriptor (11 words): kind, n_layers, dims[8], dtype.
    MLP: dims = F, h1, ..., 1 and n_layers = len(dims) - 1.
    LSTM: dims = F, H, 1 and n_layers = 2."""
    w = np.zeros(MODEL_WORDS, dtype=np.int32)
    w[0] = kind
    w[1] = len(dims) - 1
    assert len(dims) <= 8
    w[2:2 + len(dims)] = dims
    w[10] = dtype
    return w


# ----------------------------------------------------------------------------
# pipelines
# ----------------------------------------------------------------------------

def _finish(forward):
    """forward: list of dicts in network (input -> output) order with keys
    rec (stage record with placeholder indices) and ins (forward indices of the
    producers, -1 = pipeline input).  Returns the [S][16] int32 array in scheduling
    order (output first) with anchor / n_consumers / in0 / in1 filled in."""
    n = len(forward)
    consumers = [[] for _ in range(n)]
    for j, st in enumerate(forward):
        for p in st["ins"]:
            if p >= 0:
                consumers[p].append(j)
    out = np.zeros((n, STAGE_WORDS), dtype=np.int32)
    for j, st in enumerate(forward):
        rec = list(st["rec"])
        sched = n - 1 - j
        cons = [n - 1 - c for c in consumers[j]]
        rec[8] = min(cons) if cons else -1
        rec[9] = len(cons)
        ins = [(n - 1 - p) if p >= 0 else -1 for p in st["ins"]] + [-1, -1]
        rec[10], rec[11] = ins[0], ins[1]
        out[sched] = rec
    return out


def tiny_conv_relu(order="output_first"):
    """conv3x3 (8->8 channels, 16x16, stride 1) followed by ReLU, fp32 elements.
    order='output_first' lists ReLU as L_1 and the conv as L_2 (anchor = ReLU).
    order='input_first' lists the conv first and gives the ReLU the conv as anchor,
    which lets the ReLU be fused (INLINE) into the loop nest scheduled before it."""
    conv = stage_record(CONV, 16, 16, 8, RC=8, KH=3, KW=3, stride=1)
    relu = stage_record(POINTWISE, 16, 16, 8)
    if order == "output_first":
        return _finish([dict(rec=conv, ins=[-1]), dict(rec=relu, ins=[0])])
    out = np.zeros((2, STAGE_WORDS), dtype=np.int32)
    conv[8], conv[9], conv[10] = -1, 1, -1
    relu[8], relu[9], relu[10] = 0, 1, 0
    out[0], out[1] = conv, relu
    return out


def tiny_space(F=64):
    f = [1, 2, 4, 8, 16]
    return make_space(f, f, f, ALL_PERMS, 2, 2, [ROOT, INLINE], 1, F)


def resnet18_shaped(base=64, res=56):
    """20 stages in four groups of (conv3x3 -> ReLU -> conv3x3 ; conv1x1 shortcut ;
    add).  Channels base..8*base, resolution res..res/8, batch 1."""
    fwd = []
    cin, hin, src = base, res, -1
    for g in range(4):
        C = base << g
        s = 1 if g == 0 else 2
        H = (hin + s - 1) // s
        a = len(fwd)
        fwd.append(dict(rec=stage_record(CONV, H, H, C, RC=cin, KH=3, KW=3, stride=s), ins=[src]))
        fwd.append(dict(rec=stage_record(POINTWISE, H, H, C), ins=[a]))
        fwd.append(dict(rec=stage_record(CONV, H, H, C, RC=C, KH=3, KW=3, stride=1), ins=[a + 1]))
        fwd.append(dict(rec=stage_record(CONV, H, H, C, RC=cin, KH=1, KW=1, stride=s), ins=[src]))
        fwd.append(dict(rec=stage_record(ADD, H, H, C), ins=[a + 2, a + 3]))
        src, cin, hin = a + 4, C, H
    return _finish(fwd)


def resnet18_space(F=256):
    return make_space([1, 2, 4, 8], [1, 2, 4, 8], [1, 4, 8, 16], XC_INNER_PERMS,
                      2, 2, [ROOT, L1, L2, INLINE], 1, F)


def resnet18_batch(B, seed=2):
    """[B][20][16] pipelines: b = 0 has the standard shapes (64..512 channels,
    56x56..7x7); the others draw width and resolution from a seeded generator, as
    a stand-in for scheduling a set of different networks at once."""
    rng = np.random.default_rng(seed)
    out = np.zeros((B, 20, STAGE_WORDS), dtype=np.int32)
    for b in range(B):
        if b == 0:
            base, res = 64, 56
        else:
            base = int(rng.choice([32, 48, 64, 80, 96, 128]))
            res = int(rng.choice([28, 40, 56, 64, 72, 96]))
        out[b] = resnet18_shaped(base, res)
    return out


def mobilenetv2_shaped():
    """100 stages: 20 inverted-residual-shaped blocks of (1x1 expand -> ReLU ->
    depthwise 3x3 -> ReLU -> 1x1 project), 112x112..7x7, 16..320 channels, batch 1,
    as a plain chain (every stage has one consumer)."""
    cfg = [(112, 16, 2), (56, 24, 3), (28, 32, 3), (14, 64, 4), (14, 96, 3), (7, 160, 3), (7, 320, 2)]
    fwd = []
    cin, hin, src = 32, 112, -1
    first = True
    for (H, C, nb) in cfg:
        for k in range(nb):
            t = 1 if first else 6
            s = 2 if (k == 0 and H != hin) else 1
            ce = t * cin
            a = len(fwd)
            fwd.append(dict(rec=stage_record(CONV, hin, hin, ce, RC=cin), ins=[src]))
            fwd.append(dict(rec=stage_record(POINTWISE, hin, hin, ce), ins=[a]))
            fwd.append(dict(rec=stage_record(DWCONV, H, H, ce, RC=1, KH=3, KW=3, stride=s), ins=[a + 1]))
            fwd.append(dict(rec=stage_record(POINTWISE, H, H, ce), ins=[a + 2]))
            fwd.append(dict(rec=stage_record(CONV, H, H, C, RC=ce), ins=[a + 3]))
            src, cin, hin, first = a + 4, C, H, False
    return _finish(fwd)


def mobilenetv2_space(F=256):
    return make_space([1, 2, 4, 8], [1, 2, 4, 8], [1, 2, 4, 8, 16, 32, 64, 128],
                      XC_INNER_PERMS, 2, 2, [ROOT, L1, L2, INLINE], 2, F)


def random_pipeline(S, seed, max_hw=24, max_c=32):
    """Small random chain / diamond pipelines for property tests."""
    rng = np.random.default_rng(seed)
    fwd = []
    src, cin = -1, int(rng.integers(1, max_c + 1))
    hw = int(rng.integers(3, max_hw + 1))
    for j in range(S):
        kind = int(rng.choice([CONV, DWCONV, POINTWISE, ADD]))
        if kind == ADD and (j < 2 or src < 1):
            kind = POINTWISE
        if kind == CONV:
            k = int(rng.choice([1, 3, 5]))
            s = int(rng.choice([1, 2]))
            C = int(rng.integers(1, max_c + 1))
            hw = (hw + s - 1) // s
            rec = stage_record(CONV, hw, max(1, hw - int(rng.integers(0, 2))), C, RC=cin, KH=k, KW=k, stride=s)
            ins = [src]
            cin = C
        elif kind == DWCONV:
            s = int(rng.choice([1, 2]))
            hw = (hw + s - 1) // s
            rec = stage_record(DWCONV, hw, hw, cin, RC=1, KH=3, KW=3, stride=s)
            ins = [src]
        elif kind == POINTWISE:
            rec = stage_record(POINTWISE, hw, hw, cin)
            ins = [src]
        else:
            rec = stage_record(ADD, hw, hw, cin)
            # second input: an earlier stage with the same shape if there is one
            other = -1
            for p in range(len(fwd) - 2, -1, -1):
                r = fwd[p]["rec"]
                if r[1] == hw and r[2] == hw and r[3] == cin:
                    other = p
                    break
            if other < 0:
                rec = stage_record(POINTWISE, hw, hw, cin)
                ins = [src]
            else:
                ins = [src, other]
        fwd.append(dict(rec=rec, ins=ins))
        src = j
    return _finish(fwd)


# ----------------------------------------------------------------------------
# value-network weights (handed to both implementations as plain fp32 arrays)
# ----------------------------------------------------------------------------

def mlp_weights(dims, seed=0, bias_std=0.0):
    """Flat fp32 blob W_1, b_1, ..., W_L, b_L with W_k[out][in] row-major,
    entries N(0, 1/fan_in); biases zero unless bias_std > 0."""
    rng = np.random.default_rng(seed)
    parts = []
    for k in range(len(dims) - 1):
        fin, fout = dims[k], dims[k + 1]
        W = rng.standard_normal((fout, fin)) / np.sqrt(fin)
        b = rng.standard_normal(fout) * bias_std if bias_std > 0 else np.zeros(fout)
        parts += [W.reshape(-1), b]
    return np.concatenate(parts).astype(np.float32)


def lstm_weights(F, H, seed=0, bias_std=0.0):
    """Flat fp32 blob W_ih[4H][F], W_hh[4H][H], b_ih[4H], b_hh[4H], w_head[H],
    b_head[1]; the four row blocks are the gates in the order i, f, g, o."""
    rng = np.random.default_rng(seed)
    Wih = rng.standard_normal((4 * H, F)) / np.sqrt(F)
    Whh = rng.standard_normal((4 * H, H)) / np.sqrt(H)
    if bias_std > 0:
        bih = rng.standard_normal(4 * H) * bias_std
        bhh = rng.standard_normal(4 * H) * bias_std
        bhead = rng.standard_normal(1) * bias_std
    else:
        bih, bhh, bhead = np.zeros(4 * H), np.zeros(4 * H), np.zeros(1)
    wh = rng.standard_normal(H) / np.sqrt(H)
    return np.concatenate([Wih.reshape(-1), Whh.reshape(-1), bih, bhh, wh, bhead]).astype(np.float32)


def mlp_param_count(dims):
    return sum(dims[k] * dims[k + 1] + dims[k + 1] for k in range(len(dims) - 1))


def lstm_param_count(F, H):
    return 4 * H * F + 4 * H * H + 8 * H + H + 1


# ----------------------------------------------------------------------------
# raw inputs for the scoring-only workloads
# ----------------------------------------------------------------------------

def raw_feature_group(g, F=256, group=4096, seed=3, max_log2=20.0):
    """[F][group] int32 block of raw feature values floor(2^u), u ~ U[0, max_log2),
    for candidate group g.  Groups are seeded one by one so that a sample of groups
    can be regenerated without the whole matrix."""
    rng = np.random.default_rng([seed, g])
    u = rng.random((F, group)) * max_log2
    return np.floor(np.exp2(u)).astype(np.int32)


def raw_feature_matrix(n_groups, F=256, group=4096, seed=3, out=None):
    """[F][n_groups*group] int32, feature-major; column block g is raw_feature_group(g)."""
    if out is None:
        out = np.empty((F, n_groups * group), dtype=np.int32)
    for g in range(n_groups):
        out[:, g * group:(g + 1) * group] = raw_feature_group(g, F, group, seed)
    return out


def feature_sequences(first, count, T=50, F=128, seed=4, max_log2=20.0):
    """[count][T][F] bf16 bit patterns (uint16) of values u ~ U[0, max_log2): per-stage
    feature sequences already on the normalised (log2) scale.  Sequence n is seeded
    by (seed, n // 256) so a sample can be regenerated on its own."""
    import torch
    assert first % 256 == 0 and count % 256 == 0
    out = np.empty((count, T, F), dtype=np.uint16)
    for k in range(count // 256):
        rng = np.random.default_rng([seed, first // 256 + k])
        u = (rng.random((256, T, F)) * max_log2).astype(np.float32)
        b = torch.from_numpy(u).to(torch.bfloat16).view(torch.int16).numpy()
        out[k * 256:(k + 1) * 256] = b.view(np.uint16)
    return out
