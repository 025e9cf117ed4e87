"""ctypes wrapper around the CPU checker ``vf_oracle.c``.

TEST INFRASTRUCTURE: used by the tests, the smoke check and the benchmark's CPU
baseline only.  It does not import the GPU package and shares nothing with it.
Arrays are numpy; records are flat int32 arrays whose layout is fixed by the C
structs in ``vf_oracle.c``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vf_oracle.c")
# OVF_LIB: another build of the same source (the sanitizer build of the CPU tests) to load instead
_LIB = os.environ.get("OVF_LIB") or os.path.join(_HERE, "libvf_oracle.so")

OK, EINVAL, ESTATE, ENOMEM = 0, -1, -2, -3

VFUN = C.CFUNCTYPE(C.c_double, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32))


def build(force=True):
    """Compile the checker with gcc (no fast-math, no contraction, OpenMP)."""
    if os.environ.get("OVF_LIB"):
        return _LIB          # somebody else's build: taken as it is
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math",
           "-ffp-contract=off", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        L = C.CDLL(_LIB)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.ovf_dense_count.restype = i64
        L.ovf_dense_count.argtypes = [vp]
        L.ovf_padded_count.restype = i64
        L.ovf_padded_count.argtypes = [vp]
        L.ovf_states.argtypes = [vp, i32, vp, vp, i32, vp, vp]
        L.ovf_enumerate.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp]
        L.ovf_featurize.argtypes = [vp, i32, vp, vp, i32, vp]
        L.ovf_sequences.argtypes = [vp, i32, vp, vp, i32, vp, vp]
        L.ovf_plog2.restype = C.c_float
        L.ovf_plog2.argtypes = [i32]
        L.ovf_bf16_round.restype = C.c_float
        L.ovf_bf16_round.argtypes = [C.c_float]
        L.ovf_score_mlp.argtypes = [vp, vp, vp, i64, i64, vp]
        L.ovf_score_lstm.argtypes = [vp, vp, vp, i64, i32, vp]
        L.ovf_argmin.argtypes = [vp, vp, i64, i32, vp, vp]
        L.ovf_greedy.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
        L.ovf_philox4x32_10.argtypes = [vp, vp, vp]
        L.ovf_noise.restype = C.c_float
        L.ovf_noise.argtypes = [C.c_uint64, i32, i32, i32]
        L.ovf_rollouts.argtypes = [vp, i32, vp, vp, vp, C.c_float, C.c_uint64, i32, i32, vp, vp, vp, vp]
        L.ovf_decision_scores.argtypes = [vp, i32, vp, vp, vp, vp, i32, C.c_float, C.c_uint64, i32, vp, vp]
        L.ovf_beam.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
        L.ovf_num_threads.restype = i32
        L.ovf_set_num_threads.argtypes = [C.c_int]
        L.ovf_set_num_threads.restype = None
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.int32)
    if shape is not None:
        a = a.reshape(shape)
    return a


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__({EINVAL: "invalid argument", ESTATE: "invalid committed prefix",
                          ENOMEM: "out of memory"}.get(code, f"error {code}"))
        self.code = code


def _check(rc):
    if rc != OK:
        raise OracleError(rc)


def dense_count(space):
    return int(lib().ovf_dense_count(_p(_i32(space))))


def padded_count(space):
    return int(lib().ovf_padded_count(_p(_i32(space))))


def states(stages, space, cids):
    """State records [n][16] and committed core features [n][64] of a prefix."""
    stages = _i32(stages, (-1, 16)); space = _i32(space); cids = _i32(cids, (-1,))
    n = len(cids)
    st = np.zeros((max(n, 1), 16), np.int32)
    cf = np.zeros((max(n, 1), 64), np.int32)
    _check(lib().ovf_states(_p(stages), len(stages), _p(space), _p(cids), n, _p(st), _p(cf)))
    return st[:n], cf[:n]


def enumerate_candidates(stages, space, prefix_cids, stage):
    stages = _i32(stages, (-1, 16)); space = _i32(space); pre = _i32(prefix_cids, (-1,))
    assert len(pre) >= stage
    Mp = padded_count(space)
    dec = np.zeros(Mp, np.uint32); valid = np.zeros(Mp, np.uint8); nv = np.zeros(1, np.int32)
    _check(lib().ovf_enumerate(_p(stages), len(stages), _p(space), _p(pre), stage, _p(dec), _p(valid), _p(nv)))
    return dec, valid, int(nv[0])


def featurize(stages, space, prefix_cids, stage):
    """[F][M_pad] int32 features of every candidate state of decision `stage`."""
    stages = _i32(stages, (-1, 16)); space = _i32(space); pre = _i32(prefix_cids, (-1,))
    assert len(pre) >= stage
    Mp = padded_count(space)
    feat = np.empty((int(space[64]), Mp), np.int32)
    _check(lib().ovf_featurize(_p(stages), len(stages), _p(space), _p(pre), stage, _p(feat)))
    return feat


def sequences(stages, space, prefix_cids, stage):
    """Sequence form of every candidate state of decision `stage`: (x [M][S][64] uint16 bf16
    bit patterns, valid [M] uint8)."""
    stages = _i32(stages, (-1, 16)); space = _i32(space); pre = _i32(prefix_cids, (-1,))
    assert len(pre) >= stage
    M, S = dense_count(space), len(stages)
    x = np.empty((M, S, 64), np.uint16); valid = np.empty(M, np.uint8)
    _check(lib().ovf_sequences(_p(stages), S, _p(space), _p(pre), stage, _p(x), _p(valid)))
    return x, valid


def plog2(x):
    L = lib()
    x = np.asarray(x, dtype=np.int32)
    return np.array([L.ovf_plog2(int(v)) for v in x.reshape(-1)], np.float32).reshape(x.shape)


def bf16_round(v):
    L = lib()
    v = np.asarray(v, dtype=np.float32)
    return np.array([L.ovf_bf16_round(float(t)) for t in v.reshape(-1)], np.float32).reshape(v.shape)


def score_mlp(model, weights, x, M=None):
    """x: [F][ld] int32 raw features; returns float32 scores of the first M columns."""
    model = _i32(model); weights = np.ascontiguousarray(weights, np.float32)
    x = _i32(x); assert x.ndim == 2
    ld = x.shape[1]
    M = ld if M is None else M
    out = np.empty(M, np.float32)
    _check(lib().ovf_score_mlp(_p(model), _p(weights), _p(x), ld, M, _p(out)))
    return out


def score_lstm(model, weights, x):
    """x: [B][T][F] uint16 bf16 bit patterns; returns float32 scores [B]."""
    model = _i32(model); weights = np.ascontiguousarray(weights, np.float32)
    x = np.ascontiguousarray(x, np.uint16); assert x.ndim == 3
    B, T, F = x.shape
    assert F == int(model[2])
    out = np.empty(B, np.float32)
    _check(lib().ovf_score_lstm(_p(model), _p(weights), _p(x), B, T, _p(out)))
    return out


def argmin(scores, valid=None, group=0):
    scores = np.ascontiguousarray(scores, np.float32)
    M = len(scores)
    if valid is not None:
        valid = np.ascontiguousarray(valid, np.uint8); assert len(valid) >= M
    ng = 1 if group == 0 else (M + group - 1) // group
    bi = np.zeros(max(ng, 1), np.int32); bv = np.zeros(max(ng, 1), np.float32)
    _check(lib().ovf_argmin(_p(scores), _p(valid), M, group, _p(bi), _p(bv)))
    return bi[:ng], bv[:ng]


def greedy(stages, space, model=None, weights=None, vfun=None, first=0, last=None,
           prefix_cids=None, forced=None):
    """Algorithm 1.  Returns dict(cids, values, top2, states, n_evals)."""
    stages = _i32(stages, (-1, 16)); space = _i32(space)
    S = len(stages)
    last = S - 1 if last is None else last
    cids = np.full(S, -1, np.int32)
    if first > 0:
        cids[:first] = _i32(prefix_cids)[:first]
    values = np.full(S, np.inf, np.float32); top2 = np.full(S, np.inf, np.float32)
    st = np.zeros((S, 16), np.int32); ne = np.zeros(1, np.int64)
    cb = VFUN(vfun) if vfun is not None else None
    if model is not None:
        model = _i32(model); weights = np.ascontiguousarray(weights, np.float32)
    if forced is not None:
        forced = _i32(forced); assert len(forced) == S
    rc = lib().ovf_greedy(_p(stages), S, _p(space), _p(model), _p(weights),
                          C.cast(cb, C.c_void_p) if cb is not None else None, None,
                          first, last, _p(forced), _p(cids), _p(values), _p(top2), _p(st), _p(ne))
    _check(rc)
    return dict(cids=cids, values=values, top2=top2, states=st, n_evals=int(ne[0]))


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, np.uint32); k = np.asarray(key, np.uint32); out = np.zeros(4, np.uint32)
    lib().ovf_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def noise(seed, rollout, stage, cid):
    return float(lib().ovf_noise(seed, rollout, stage, cid))


def rollouts(stages, space, model, weights, eps, seed, n_rollouts, first_rollout=0, forced=None):
    """n_rollouts noisy greedy schedules.  Returns dict(cids, values, top2), each [n][S]."""
    stages = _i32(stages, (-1, 16)); space = _i32(space); model = _i32(model)
    weights = np.ascontiguousarray(weights, np.float32)
    S = len(stages)
    cids = np.full((n_rollouts, S), -1, np.int32)
    values = np.full((n_rollouts, S), np.inf, np.float32); top2 = np.full((n_rollouts, S), np.inf, np.float32)
    if forced is not None:
        forced = _i32(forced, (n_rollouts, S))
    _check(lib().ovf_rollouts(_p(stages), S, _p(space), _p(model), _p(weights), C.c_float(eps), seed,
                              first_rollout, n_rollouts, _p(forced), _p(cids), _p(values), _p(top2)))
    return dict(cids=cids, values=values, top2=top2)


def decision_scores(stages, space, model, weights, prefix_cids, stage, eps=0.0, seed=0, rollout=0):
    """(scores [M] float32, valid [M] bool) as the scan of decision `stage` sees them after the
    committed prefix, exploration noise of `rollout` included when eps != 0."""
    stages = _i32(stages, (-1, 16)); space = _i32(space); model = _i32(model)
    weights = np.ascontiguousarray(weights, np.float32); pre = _i32(prefix_cids, (-1,))
    assert len(pre) >= stage
    M = dense_count(space)
    sc = np.empty(M, np.float32); ok = np.zeros(M, np.uint8)
    _check(lib().ovf_decision_scores(_p(stages), len(stages), _p(space), _p(model), _p(weights), _p(pre), stage,
                                     C.c_float(eps), seed, rollout, _p(sc), _p(ok)))
    return sc, ok != 0


def beam(stages, space, width, model=None, weights=None, vfun=None):
    """Beam search of the given width guided by V.  Returns dict(cids [width][S],
    values [width][S], n_beams, n_evals); width = 1 is the greedy scan."""
    stages = _i32(stages, (-1, 16)); space = _i32(space)
    S = len(stages)
    cids = np.full((width, S), -1, np.int32); values = np.full((width, S), np.inf, np.float32)
    nb = np.zeros(1, np.int32); ne = np.zeros(1, np.int64)
    cb = VFUN(vfun) if vfun is not None else None
    if model is not None:
        model = _i32(model); weights = np.ascontiguousarray(weights, np.float32)
    _check(lib().ovf_beam(_p(stages), S, _p(space), _p(model), _p(weights),
                          C.cast(cb, C.c_void_p) if cb is not None else None, None, width,
                          _p(cids), _p(values), _p(nb), _p(ne)))
    return dict(cids=cids, values=values, n_beams=int(nb[0]), n_evals=int(ne[0]))


def num_threads():
    return int(lib().ovf_num_threads())


def set_num_threads(n):
    """Threads used by the loops over candidates from now on (for timing)."""
    lib().ovf_set_num_threads(int(n))
