"""Thin ctypes binding of libvf.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/vf.h) and
takes / returns torch tensors on the context's GPU.  PyTorch is used for device
memory and for the stream; every step of the scheduler runs in the library's HIP
kernels.  There is no CPU fallback: if libvf.so is missing or cannot be loaded the
import of this module's library raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvf.so")

VF_OK, VF_EINVAL, VF_ESTATE, VF_ENOMEM, VF_EHIP = 0, -1, -2, -3, -4
VF_X_RAW_I32, VF_X_SEQ_BF16 = 0, 1

EXPORTS = [
    "vf_create", "vf_destroy", "vf_set_space", "vf_set_pipeline", "vf_set_model", "vf_reset_state",
    "vf_set_state", "vf_n_scheduled", "vf_dense_count", "vf_padded_count", "vf_enumerate",
    "vf_featurize", "vf_score", "vf_score_static", "vf_score_static_max", "vf_argmin_step", "vf_greedy_schedule", "vf_beam_search", "vf_set_noise", "vf_strerror",
    "vf_last_hip_error", "vf_timer_start", "vf_timer_stop", "vf_timer_elapsed_ms",
    "vf_profile_enable", "vf_profile_read", "vf_profile_counts", "vf_set_wait_limit", "vf_sync_status",
]

_lib = None


class VfError(RuntimeError):
    def __init__(self, code, hip=0):
        msg = lib().vf_strerror(code).decode()
        if hip:
            msg += f" (hip status {hip})"
        super().__init__(msg)
        self.code = code
        self.hip = hip


def lib():
    """Loads libvf.so (built in-tree by paper_2011_14486_amd.build).  Raises if absent."""
    global _lib
    if _lib is None:
        # PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  It has to be in the
        # process first so that libvf.so binds to that same runtime: streams and device
        # pointers are only meaningful within one runtime instance.
        import torch  # noqa: F401
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with paper_2011_14486_amd.build.build_lib(); "
                              "there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.vf_create.argtypes = [C.POINTER(vp), C.c_int, vp]
        L.vf_destroy.argtypes = [vp]
        L.vf_destroy.restype = None
        L.vf_set_space.argtypes = [vp, vp]
        L.vf_set_pipeline.argtypes = [vp, vp, C.c_int, C.c_int]
        L.vf_set_model.argtypes = [vp, vp, vp, C.c_size_t]
        L.vf_reset_state.argtypes = [vp]
        L.vf_set_state.argtypes = [vp, vp, C.c_int]
        L.vf_n_scheduled.argtypes = [vp]
        L.vf_dense_count.argtypes = [vp]
        L.vf_dense_count.restype = i64
        L.vf_padded_count.argtypes = [vp]
        L.vf_padded_count.restype = i64
        L.vf_enumerate.argtypes = [vp, C.c_int, vp, vp, vp]
        L.vf_featurize.argtypes = [vp, C.c_int, vp]
        L.vf_score.argtypes = [vp, vp, i32, i64, i64, i32, vp, vp, vp]
        L.vf_score_static.argtypes = [vp, vp, i32, i64, i64, i32, vp, vp, vp]
        L.vf_score_static_max.argtypes = [vp]
        L.vf_score_static_max.restype = i64
        L.vf_argmin_step.argtypes = [vp, C.c_int, C.c_int, vp, vp]
        L.vf_greedy_schedule.argtypes = [vp, C.c_int, C.c_int, vp, vp, vp]
        L.vf_set_noise.argtypes = [vp, C.c_float, C.c_uint64, i32]
        L.vf_beam_search.argtypes = [vp, C.c_int, C.c_int, vp, vp, vp, vp]
        L.vf_strerror.argtypes = [C.c_int]
        L.vf_strerror.restype = C.c_char_p
        L.vf_last_hip_error.argtypes = [vp]
        L.vf_timer_start.argtypes = [vp]
        L.vf_timer_stop.argtypes = [vp]
        L.vf_timer_elapsed_ms.argtypes = [vp, C.POINTER(C.c_float)]
        L.vf_profile_enable.argtypes = [vp, C.c_int]
        L.vf_profile_read.argtypes = [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(i64)]
        L.vf_profile_counts.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
        L.vf_set_wait_limit.argtypes = [vp, C.c_uint]
        L.vf_sync_status.argtypes = [vp]
        _lib = L
    return _lib


def _check(ctx, rc):
    if rc != VF_OK:
        raise VfError(rc, lib().vf_last_hip_error(ctx.handle) if ctx is not None and ctx.handle else 0)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _np32(a, n=None):
    a = np.ascontiguousarray(a, dtype=np.int32)
    if n is not None:
        assert a.size == n, (a.size, n)
    return a


class Context:
    """Owns one vf_ctx.  Holds the torch device and stream the context was made on."""

    def __init__(self, device=0, stream=None):
        import torch
        self.torch = torch
        self.device = torch.device("cuda", device)
        with torch.cuda.device(self.device):
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        rc = lib().vf_create(C.byref(h), device, C.c_void_p(self.stream.cuda_stream))
        self.handle = h if rc == VF_OK else None
        _check(None, rc)
        self.F = self.S = self.B = 0

    def close(self):
        if self.handle:
            lib().vf_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def empty(self, shape, dtype):
        return self.torch.empty(shape, dtype=dtype, device=self.device)


def vf_create(device=0, stream=None):
    return Context(device, stream)


def vf_destroy(ctx):
    ctx.close()


def vf_set_space(ctx, space):
    s = _np32(space, 65)
    _check(ctx, lib().vf_set_space(ctx.handle, s.ctypes.data_as(C.c_void_p)))
    ctx.F = int(s[64])


def vf_set_pipeline(ctx, stages):
    """stages: [S][16] (one problem) or [B][S][16] int32."""
    st = _np32(stages)
    if st.ndim == 2:
        st = st[None]
    assert st.ndim == 3 and st.shape[2] == 16
    _check(ctx, lib().vf_set_pipeline(ctx.handle, st.ctypes.data_as(C.c_void_p), st.shape[1], st.shape[0]))
    ctx.B, ctx.S = st.shape[0], st.shape[1]


def vf_set_model(ctx, model, weights):
    """model: 11-word record; weights: fp32 numpy array or CUDA tensor (flat blob)."""
    torch = ctx.torch
    m = _np32(model, 11)
    if not isinstance(weights, torch.Tensor):
        weights = torch.from_numpy(np.ascontiguousarray(weights, np.float32))
    w = weights.to(device=ctx.device, dtype=torch.float32).contiguous()
    ctx.stream.wait_stream(torch.cuda.current_stream(ctx.device))
    _check(ctx, lib().vf_set_model(ctx.handle, m.ctypes.data_as(C.c_void_p), _ptr(w), w.numel()))


def vf_reset_state(ctx):
    _check(ctx, lib().vf_reset_state(ctx.handle))


def vf_set_state(ctx, cids):
    c = _np32(cids)
    if c.ndim == 1:
        c = c[None]
    assert c.shape[0] == ctx.B
    _check(ctx, lib().vf_set_state(ctx.handle, c.ctypes.data_as(C.c_void_p) if c.size else None, c.shape[1]))


def vf_n_scheduled(ctx):
    return int(lib().vf_n_scheduled(ctx.handle))


def vf_dense_count(ctx):
    return int(lib().vf_dense_count(ctx.handle))


def vf_padded_count(ctx):
    return int(lib().vf_padded_count(ctx.handle))


def vf_enumerate(ctx, stage):
    """Returns (dec int32-viewed-as-uint32 [B][M_pad], valid uint8 [B][M_pad], n_valid int32 [B])."""
    torch = ctx.torch
    Mp = vf_padded_count(ctx)
    dec = ctx.empty((ctx.B, Mp), torch.int32)
    valid = ctx.empty((ctx.B, Mp), torch.uint8)
    nv = ctx.empty((ctx.B,), torch.int32)
    _check(ctx, lib().vf_enumerate(ctx.handle, stage, _ptr(dec), _ptr(valid), _ptr(nv)))
    return dec, valid, nv


def vf_featurize(ctx, stage, out=None):
    """Returns feat int32 [B][F][M_pad]."""
    torch = ctx.torch
    Mp = vf_padded_count(ctx)
    if out is None:
        out = ctx.empty((ctx.B, ctx.F, Mp), torch.int32)
    assert out.is_contiguous() and out.numel() == ctx.B * ctx.F * Mp and out.dtype == torch.int32
    _check(ctx, lib().vf_featurize(ctx.handle, stage, _ptr(out)))
    return out


def vf_score(ctx, x, x_kind=VF_X_RAW_I32, M=None, group=0, want_scores=True, want_min=True):
    """x: int32 [F][ld] (VF_X_RAW_I32) or bf16 [M][T][F] (VF_X_SEQ_BF16) CUDA tensor.
    Returns (scores float32 [M] or None, best_idx int32 [groups] or None, best_val float32 or None)."""
    torch = ctx.torch
    assert x.is_cuda and x.is_contiguous()
    if x_kind == VF_X_RAW_I32:
        assert x.dtype == torch.int32 and x.dim() == 2
        ld = x.shape[1]
        M = ld if M is None else M
    else:
        assert x.dtype == torch.bfloat16 and x.dim() == 3
        M = x.shape[0] if M is None else M
        ld = x.shape[1]
    ng = 1 if group == 0 else max((M + group - 1) // group, 1)
    scores = ctx.empty((M,), torch.float32) if want_scores else None
    bi = ctx.empty((ng,), torch.int32) if want_min else None
    bv = ctx.empty((ng,), torch.float32) if want_min else None
    _check(ctx, lib().vf_score(ctx.handle, _ptr(x), x_kind, M, ld, group, _ptr(scores), _ptr(bi), _ptr(bv)))
    return scores, bi, bv


def vf_score_static(ctx, x, x_kind=VF_X_RAW_I32, M=None, group=0, out=None):
    """vf_score through the entry point that allocates nothing.  out = (scores or None, best_idx,
    best_val): tensors the caller made beforehand (this wrapper makes them when out is None, which
    is an allocation by torch, outside the library call)."""
    torch = ctx.torch
    assert x.is_cuda and x.is_contiguous()
    if x_kind == VF_X_RAW_I32:
        ld = x.shape[1]
        M = ld if M is None else M
    else:
        M = x.shape[0] if M is None else M
        ld = x.shape[1]
    ng = 1 if group == 0 else max((M + group - 1) // group, 1)
    if out is None:
        out = (ctx.empty((M,), torch.float32), ctx.empty((ng,), torch.int32), ctx.empty((ng,), torch.float32))
    scores, bi, bv = out
    _check(ctx, lib().vf_score_static(ctx.handle, _ptr(x), x_kind, M, ld, group, _ptr(scores), _ptr(bi), _ptr(bv)))
    return scores, bi, bv


def vf_score_static_max(ctx):
    return int(lib().vf_score_static_max(ctx.handle))


def vf_argmin_step(ctx, stage, commit=True):
    torch = ctx.torch
    bc = ctx.empty((ctx.B,), torch.int32)
    bv = ctx.empty((ctx.B,), torch.float32)
    _check(ctx, lib().vf_argmin_step(ctx.handle, stage, 1 if commit else 0, _ptr(bc), _ptr(bv)))
    return bc, bv


def vf_greedy_schedule(ctx, first=0, last=None, out=None):
    """Returns (states int32 [B][S][16], cids int32 [B][S], values float32 [B][S])."""
    torch = ctx.torch
    last = ctx.S - 1 if last is None else last
    if out is None:
        out = (ctx.empty((ctx.B, ctx.S, 16), torch.int32), ctx.empty((ctx.B, ctx.S), torch.int32),
               ctx.empty((ctx.B, ctx.S), torch.float32))
    st, cids, vals = out
    _check(ctx, lib().vf_greedy_schedule(ctx.handle, first, last, _ptr(st), _ptr(cids), _ptr(vals)))
    return st, cids, vals


def vf_set_noise(ctx, eps, seed=0, first_rollout=0):
    _check(ctx, lib().vf_set_noise(ctx.handle, C.c_float(eps), seed, first_rollout))


def vf_beam_search(ctx, first=0, last=None):
    """Beam search of width ctx.B.  Returns (states [B][S][16], cids [B][S], values [B][S], n_beams [1])."""
    torch = ctx.torch
    last = ctx.S - 1 if last is None else last
    st = ctx.empty((ctx.B, ctx.S, 16), torch.int32)
    cids = ctx.empty((ctx.B, ctx.S), torch.int32)
    vals = ctx.empty((ctx.B, ctx.S), torch.float32)
    nb = ctx.empty((1,), torch.int32)
    _check(ctx, lib().vf_beam_search(ctx.handle, first, last, _ptr(st), _ptr(cids), _ptr(vals), _ptr(nb)))
    return st, cids, vals, nb


def vf_timer_start(ctx):
    _check(ctx, lib().vf_timer_start(ctx.handle))


def vf_timer_stop(ctx):
    _check(ctx, lib().vf_timer_stop(ctx.handle))


def vf_timer_elapsed_ms(ctx):
    ms = C.c_float()
    _check(ctx, lib().vf_timer_elapsed_ms(ctx.handle, C.byref(ms)))
    return float(ms.value)


VF_PROF_FEATURIZE, VF_PROF_SCORE, VF_PROF_COMMIT = 0, 1, 2


def vf_profile_enable(ctx, enable=True):
    _check(ctx, lib().vf_profile_enable(ctx.handle, 1 if enable else 0))


def vf_profile_read(ctx, which):
    """Returns (total milliseconds, launches) of one kernel kind since the last read."""
    ms, n = C.c_double(), C.c_int64()
    _check(ctx, lib().vf_profile_read(ctx.handle, which, C.byref(ms), C.byref(n)))
    return float(ms.value), int(n.value)


def vf_set_wait_limit(ctx, rounds):
    """Bound (polling rounds) of the waits between workgroups that share a problem in vf_greedy_schedule."""
    _check(ctx, lib().vf_set_wait_limit(ctx.handle, int(rounds)))


def vf_sync_status(ctx):
    """Waits for the context's stream; raises VfError(VF_ESTATE) if the last whole-schedule launch gave
    up a wait (its layers have then been run again per layer where the state was still there)."""
    _check(ctx, lib().vf_sync_status(ctx.handle))


def vf_profile_counts(ctx):
    """Returns (ids pushed through V, valid candidates among them) by the fused step since the last call."""
    a, b = C.c_int64(), C.c_int64()
    _check(ctx, lib().vf_profile_counts(ctx.handle, C.byref(a), C.byref(b)))
    return int(a.value), int(b.value)
