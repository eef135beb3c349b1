"""ctypes front end of the CPU oracle (oracle/cocodc_ref.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  The product package never imports this module, and this module never
imports the product package.  It only marshals numpy arrays into the C functions; all
arithmetic lives in cocodc_ref.cpp.

All arrays are host numpy arrays: float32 and C-contiguous for parameter buffers (updated
in place where the C function updates in place), int64 for I_p / t_b, float64 for scores.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libcocodc_ref.so")
_lib = None


class Fragment(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("length", C.c_uint64)]


class HParams(C.Structure):
    _fields_ = [
        ("tau", C.c_int32), ("H", C.c_int32),
        ("lambda_", C.c_double), ("eta", C.c_double), ("mu", C.c_double),
        ("nesterov", C.c_int32), ("drift_sign", C.c_int32),
        ("score_src", C.c_int32), ("norm_kind", C.c_int32),
        ("merge_mode", C.c_int32), ("alpha", C.c_double),
        ("delta_src", C.c_int32), ("pg_format", C.c_int32),
    ]


class Segment(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("length", C.c_uint64), ("fragment", C.c_int32), ("reserved", C.c_int32)]


class Shadow(C.Structure):
    _fields_ = [("theta_m", C.c_void_p), ("theta_g", C.c_void_p), ("momentum", C.c_void_p)]


def hparams(tau, H, lam=0.5, eta=0.7, mu=0.9, nesterov=1, drift_sign=1, score_src=0, norm_kind=2,
            merge_mode=0, alpha=1.0, delta_src=0, pg_format=0):
    return HParams(int(tau), int(H), float(lam), float(eta), float(mu), int(nesterov),
                   int(drift_sign), int(score_src), int(norm_kind), int(merge_mode), float(alpha),
                   int(delta_src), int(pg_format))


def lib():
    """Load (building it first if it is missing) the oracle shared library."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _build
            _build.build(force=True)
        _lib = C.CDLL(_LIB_PATH)
        for name in ("pseudograd", "outer_nesterov", "delay_compensate", "fragment_scores",
                     "select_fragments", "sync_step", "sync_step_mt", "sync_plan",
                     "fragment_scores_segmented", "sync_step_segmented", "pseudograd_bf16", "sync_step_bf16",
                     "select_fragments_bytes", "sync_event", "sync_step_bf16_segmented", "sync_event_bf16", "sync_event_segmented", "sync_event_bf16_segmented"):
            getattr(_lib, "cocodc_ref_" + name).restype = C.c_int
        _lib.cocodc_ref_round_bf16.restype = C.c_uint16
        _lib.cocodc_ref_round_bf16.argtypes = [C.c_double]
        _lib.cocodc_ref_widen_bf16.restype = C.c_double
        _lib.cocodc_ref_widen_bf16.argtypes = [C.c_uint16]
        _lib.cocodc_ref_round_f16.restype = C.c_uint16
        _lib.cocodc_ref_round_f16.argtypes = [C.c_double]
        _lib.cocodc_ref_widen_f16.restype = C.c_double
        _lib.cocodc_ref_widen_f16.argtypes = [C.c_uint16]
    return _lib


def _frag_array(frags):
    arr = (Fragment * len(frags))()
    for i, (off, length) in enumerate(frags):
        arr[i].offset = int(off)
        arr[i].length = int(length)
    return arr


def _f32(a, allow_none=False):
    if a is None:
        assert allow_none
        return None
    assert isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, C.c_void_p(a.ctypes.data)


def pseudograd(frags, theta_g_snap, theta_m, delta_m_out, theta_m_send_out=None):
    n = theta_m.size
    return lib().cocodc_ref_pseudograd(_frag_array(frags), C.c_int32(len(frags)), C.c_uint64(n),
                                       _f32(theta_g_snap), _f32(theta_m), _f32(delta_m_out),
                                       _f32(theta_m_send_out, True))


def outer_nesterov(frags, theta_g, momentum, delta_g, hp):
    n = theta_g.size
    return lib().cocodc_ref_outer_nesterov(_frag_array(frags), C.c_int32(len(frags)), C.c_uint64(n),
                                           _f32(theta_g), _f32(momentum), _f32(delta_g),
                                           C.byref(hp))


def delay_compensate(frags, theta_m, theta_m_send, theta_g, hp):
    n = theta_m.size
    return lib().cocodc_ref_delay_compensate(_frag_array(frags), C.c_int32(len(frags)),
                                             C.c_uint64(n), _f32(theta_m), _f32(theta_m_send, True),
                                             _f32(theta_g), C.byref(hp))


def fragment_scores(frags, x, I_p, norm_kind=2):
    """Returns (rc, R[K], sums[K])."""
    K = len(frags)
    R = np.zeros(K, dtype=np.float64)
    S = np.zeros(K, dtype=np.float64)
    keep, ip = _i64(I_p)
    rc = lib().cocodc_ref_fragment_scores(_frag_array(frags), C.c_int32(K), C.c_uint64(x.size),
                                          _f32(x), ip, C.c_int32(norm_kind),
                                          C.c_void_p(R.ctypes.data), C.c_void_p(S.ctypes.data))
    return rc, R, S


def select_fragments(R, t_b, t_g, H, budget):
    """Returns (rc, sel[n_sel])."""
    R = np.ascontiguousarray(R, dtype=np.float64)
    K = R.size
    keep, tb = _i64(t_b)
    sel = np.full(max(K, 1), -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    rc = lib().cocodc_ref_select_fragments(C.c_int32(K), C.c_void_p(R.ctypes.data), tb,
                                           C.c_int64(t_g), C.c_int32(H), C.c_int32(budget),
                                           C.c_void_p(sel.ctypes.data), C.byref(n_sel))
    if rc != 0:
        return rc, None
    return rc, sel[:n_sel.value].copy()


def select_fragments_bytes(R, t_b, t_g, H, frag_bytes, byte_budget):
    """Returns (rc, sel[n_sel])."""
    R = np.ascontiguousarray(R, dtype=np.float64)
    K = R.size
    keep, tb = _i64(t_b)
    fb = np.ascontiguousarray(frag_bytes, dtype=np.uint64)
    sel = np.full(max(K, 1), -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    rc = lib().cocodc_ref_select_fragments_bytes(C.c_int32(K), C.c_void_p(R.ctypes.data), tb, C.c_int64(t_g),
                                                 C.c_int32(H), C.c_void_p(fb.ctypes.data), C.c_uint64(byte_budget),
                                                 C.c_void_p(sel.ctypes.data), C.byref(n_sel))
    if rc != 0:
        return rc, None
    return rc, sel[:n_sel.value].copy()


def sync_step(frags, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, t_g,
              budget, hp, shadow=False, n_threads=None):
    """Fused step, in place on theta_m / theta_g / momentum (and delta_m_out).

    Returns a dict: rc, R[K], sel[n_sel], sums[K,4] and, with shadow=True, the unrounded
    fp64 theta_m / theta_g / momentum.  n_threads selects the chunk-parallel timing variant.
    """
    K = len(frags)
    n = theta_m.size
    R = np.zeros(K, dtype=np.float64)
    sums = np.zeros((K, 4), dtype=np.float64)
    sel = np.full(K, -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    keep1, ip = _i64(I_p)
    keep2, tb = _i64(t_b)
    out = {}
    common = (_frag_array(frags), C.c_int32(K), C.c_uint64(n), _f32(theta_m), _f32(theta_m_send, True),
              _f32(theta_g), _f32(momentum), _f32(delta_g), _f32(delta_m_out, True), ip, tb,
              C.c_int64(t_g), C.c_int32(budget), C.byref(hp), C.c_void_p(R.ctypes.data),
              C.c_void_p(sel.ctypes.data), C.byref(n_sel), C.c_void_p(sums.ctypes.data))
    if n_threads is None:
        sh_ptr = None
        if shadow:
            out["theta_m64"] = np.zeros(n, dtype=np.float64)
            out["theta_g64"] = np.zeros(n, dtype=np.float64)
            out["momentum64"] = np.zeros(n, dtype=np.float64)
            sh = Shadow(out["theta_m64"].ctypes.data, out["theta_g64"].ctypes.data,
                        out["momentum64"].ctypes.data)
            sh_ptr = C.byref(sh)
        rc = lib().cocodc_ref_sync_step(*common, sh_ptr)
    else:
        rc = lib().cocodc_ref_sync_step_mt(*common, C.c_int32(n_threads))
        out["threads"] = rc
        rc = 0 if rc > 0 else rc
    out.update(rc=rc, R=R, sums=sums, sel=sel[:max(n_sel.value, 0)].copy())
    return out


def _seg_array(segs):
    arr = (Segment * max(len(segs), 1))()
    for i, (off, length, frag) in enumerate(segs):
        arr[i].offset, arr[i].length, arr[i].fragment, arr[i].reserved = int(off), int(length), int(frag), 0
    return arr


def fragment_scores_segmented(segs, K, x, I_p, norm_kind=2):
    """segs: [(offset, length, fragment), ...].  Returns (rc, R[K], sums[K])."""
    R = np.zeros(K, dtype=np.float64)
    S = np.zeros(K, dtype=np.float64)
    keep, ip = _i64(I_p)
    rc = lib().cocodc_ref_fragment_scores_segmented(_seg_array(segs), C.c_int32(len(segs)), C.c_int32(K),
                                                    C.c_uint64(x.size), _f32(x), ip, C.c_int32(norm_kind),
                                                    C.c_void_p(R.ctypes.data), C.c_void_p(S.ctypes.data))
    return rc, R, S


def sync_event(frags, recv_mask, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, t_g,
               budget, hp, R, sums=None):
    """One loop event: fused step on the fragments whose recv_mask entry has bit 0 set (True counts as 1),
    R (numpy float64, K) updated in place for them, selection over the fragments whose entry does not have
    bit 1 (in flight) set.  Returns dict rc, sel."""
    K = len(frags)
    n = theta_m.size
    assert R.dtype == np.float64 and R.size == K
    mask = np.ascontiguousarray(np.asarray(recv_mask, dtype=np.uint8))
    sel = np.full(K, -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    keep1, ip = _i64(I_p)
    keep2, tb = _i64(t_b)
    rc = lib().cocodc_ref_sync_event(
        _frag_array(frags), C.c_int32(K), C.c_uint64(n), C.c_void_p(mask.ctypes.data), _f32(theta_m),
        _f32(theta_m_send, True), _f32(theta_g), _f32(momentum), _f32(delta_g), _f32(delta_m_out, True), ip, tb,
        C.c_int64(t_g), C.c_int32(budget), C.byref(hp), C.c_void_p(R.ctypes.data), C.c_void_p(sel.ctypes.data),
        C.byref(n_sel), C.c_void_p(sums.ctypes.data) if sums is not None else None)
    return dict(rc=rc, sel=sel[:max(n_sel.value, 0)].copy())


def sync_event_segmented(segs, K, recv_mask, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b,
                         t_g, budget, hp, R, sums=None):
    """sync_event for fragments made of segments [(offset, length, fragment), ...]; R (K) updated in place."""
    n = theta_m.size
    assert R.dtype == np.float64 and R.size == K
    mask = np.ascontiguousarray(np.asarray(recv_mask, dtype=np.uint8))
    sel = np.full(K, -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    keep1, ip = _i64(I_p)
    keep2, tb = _i64(t_b)
    rc = lib().cocodc_ref_sync_event_segmented(
        _seg_array(segs), C.c_int32(len(segs)), C.c_int32(K), C.c_uint64(n), C.c_void_p(mask.ctypes.data),
        _f32(theta_m), _f32(theta_m_send, True), _f32(theta_g), _f32(momentum), _f32(delta_g),
        _f32(delta_m_out, True), ip, tb, C.c_int64(t_g), C.c_int32(budget), C.byref(hp), C.c_void_p(R.ctypes.data),
        C.c_void_p(sel.ctypes.data), C.byref(n_sel), C.c_void_p(sums.ctypes.data) if sums is not None else None)
    return dict(rc=rc, sel=sel[:max(n_sel.value, 0)].copy())


def sync_step_segmented(segs, K, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b,
                        t_g, budget, hp, shadow=False):
    """Fused step over fragments made of segments [(offset, length, fragment), ...]."""
    n = theta_m.size
    R = np.zeros(K, dtype=np.float64)
    sums = np.zeros((K, 4), dtype=np.float64)
    sel = np.full(K, -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    keep1, ip = _i64(I_p)
    keep2, tb = _i64(t_b)
    out = {}
    sh_ptr = None
    if shadow:
        out["theta_m64"] = np.zeros(n, dtype=np.float64)
        out["theta_g64"] = np.zeros(n, dtype=np.float64)
        out["momentum64"] = np.zeros(n, dtype=np.float64)
        sh = Shadow(out["theta_m64"].ctypes.data, out["theta_g64"].ctypes.data, out["momentum64"].ctypes.data)
        sh_ptr = C.byref(sh)
    rc = lib().cocodc_ref_sync_step_segmented(
        _seg_array(segs), C.c_int32(len(segs)), C.c_int32(K), C.c_uint64(n), _f32(theta_m),
        _f32(theta_m_send, True), _f32(theta_g), _f32(momentum), _f32(delta_g), _f32(delta_m_out, True), ip, tb,
        C.c_int64(t_g), C.c_int32(budget), C.byref(hp), C.c_void_p(R.ctypes.data), C.c_void_p(sel.ctypes.data),
        C.byref(n_sel), C.c_void_p(sums.ctypes.data), sh_ptr)
    out.update(rc=rc, R=R, sums=sums, sel=sel[:max(n_sel.value, 0)].copy())
    return out


def _u16(a, allow_none=False):
    if a is None:
        assert allow_none
        return None
    assert isinstance(a, np.ndarray) and a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    return C.c_void_p(a.ctypes.data)


def round_bf16(x):
    return int(lib().cocodc_ref_round_bf16(float(x)))


def widen_bf16(b):
    return float(lib().cocodc_ref_widen_bf16(int(b)))


def round_f16(x):
    return int(lib().cocodc_ref_round_f16(float(x)))


def widen_f16(b):
    return float(lib().cocodc_ref_widen_f16(int(b)))


def pseudograd_bf16(frags, theta_g_snap, theta_m, delta_m_out, theta_m_send_out=None, pg_format=0):
    """theta_m, theta_m_send_out: uint16 arrays holding bf16 bit patterns; delta_m_out: uint16 patterns of
    bf16 (pg_format 0) or IEEE binary16 (pg_format 1)."""
    return lib().cocodc_ref_pseudograd_bf16(_frag_array(frags), C.c_int32(len(frags)), C.c_uint64(theta_m.size),
                                            _f32(theta_g_snap), _u16(theta_m), _u16(delta_m_out),
                                            _u16(theta_m_send_out, True), C.c_int32(pg_format))


def sync_step_bf16(frags, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, t_g, budget, hp,
                   shadow=False):
    """Fused step with bf16 (uint16 bit patterns) theta_m / theta_m_send / delta_m_out."""
    K = len(frags)
    n = theta_m.size
    R = np.zeros(K, dtype=np.float64)
    sums = np.zeros((K, 4), dtype=np.float64)
    sel = np.full(K, -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    keep1, ip = _i64(I_p)
    keep2, tb = _i64(t_b)
    out = {}
    sh_ptr = None
    if shadow:
        out["theta_m64"] = np.zeros(n, dtype=np.float64)
        out["theta_g64"] = np.zeros(n, dtype=np.float64)
        out["momentum64"] = np.zeros(n, dtype=np.float64)
        sh = Shadow(out["theta_m64"].ctypes.data, out["theta_g64"].ctypes.data, out["momentum64"].ctypes.data)
        sh_ptr = C.byref(sh)
    rc = lib().cocodc_ref_sync_step_bf16(
        _frag_array(frags), C.c_int32(K), C.c_uint64(n), _u16(theta_m), _u16(theta_m_send, True), _f32(theta_g),
        _f32(momentum), _f32(delta_g), _u16(delta_m_out, True), ip, tb, C.c_int64(t_g), C.c_int32(budget),
        C.byref(hp), C.c_void_p(R.ctypes.data), C.c_void_p(sel.ctypes.data), C.byref(n_sel),
        C.c_void_p(sums.ctypes.data), sh_ptr)
    out.update(rc=rc, R=R, sums=sums, sel=sel[:max(n_sel.value, 0)].copy())
    return out


def sync_step_bf16_segmented(segs, K, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, t_g,
                             budget, hp):
    """sync_step_bf16 over fragments made of segments [(offset, length, fragment), ...]."""
    n = theta_m.size
    R = np.zeros(K, dtype=np.float64)
    sums = np.zeros((K, 4), dtype=np.float64)
    sel = np.full(K, -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    keep1, ip = _i64(I_p)
    keep2, tb = _i64(t_b)
    rc = lib().cocodc_ref_sync_step_bf16_segmented(
        _seg_array(segs), C.c_int32(len(segs)), C.c_int32(K), C.c_uint64(n), _u16(theta_m), _u16(theta_m_send, True),
        _f32(theta_g), _f32(momentum), _f32(delta_g), _u16(delta_m_out, True), ip, tb, C.c_int64(t_g),
        C.c_int32(budget), C.byref(hp), C.c_void_p(R.ctypes.data), C.c_void_p(sel.ctypes.data), C.byref(n_sel),
        C.c_void_p(sums.ctypes.data))
    return dict(rc=rc, R=R, sums=sums, sel=sel[:max(n_sel.value, 0)].copy())


def sync_event_bf16(frags, recv_mask, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, t_g,
                    budget, hp, R, sums=None):
    """sync_event with bf16 (uint16 bit patterns) theta_m / theta_m_send / delta_m_out; R updated in place."""
    K = len(frags)
    n = theta_m.size
    assert R.dtype == np.float64 and R.size == K
    mask = np.ascontiguousarray(np.asarray(recv_mask, dtype=np.uint8))
    sel = np.full(K, -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    keep1, ip = _i64(I_p)
    keep2, tb = _i64(t_b)
    rc = lib().cocodc_ref_sync_event_bf16(
        _frag_array(frags), C.c_int32(K), C.c_uint64(n), C.c_void_p(mask.ctypes.data), _u16(theta_m),
        _u16(theta_m_send, True), _f32(theta_g), _f32(momentum), _f32(delta_g), _u16(delta_m_out, True), ip, tb,
        C.c_int64(t_g), C.c_int32(budget), C.byref(hp), C.c_void_p(R.ctypes.data), C.c_void_p(sel.ctypes.data),
        C.byref(n_sel), C.c_void_p(sums.ctypes.data) if sums is not None else None)
    return dict(rc=rc, sel=sel[:max(n_sel.value, 0)].copy())


def sync_event_bf16_segmented(segs, K, recv_mask, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p,
                              t_b, t_g, budget, hp, R, sums=None):
    """sync_event_bf16 for fragments made of segments; R (K) updated in place."""
    n = theta_m.size
    assert R.dtype == np.float64 and R.size == K
    mask = np.ascontiguousarray(np.asarray(recv_mask, dtype=np.uint8))
    sel = np.full(K, -1, dtype=np.int32)
    n_sel = C.c_int32(-1)
    keep1, ip = _i64(I_p)
    keep2, tb = _i64(t_b)
    rc = lib().cocodc_ref_sync_event_bf16_segmented(
        _seg_array(segs), C.c_int32(len(segs)), C.c_int32(K), C.c_uint64(n), C.c_void_p(mask.ctypes.data),
        _u16(theta_m), _u16(theta_m_send, True), _f32(theta_g), _f32(momentum), _f32(delta_g), _u16(delta_m_out, True),
        ip, tb, C.c_int64(t_g), C.c_int32(budget), C.byref(hp), C.c_void_p(R.ctypes.data), C.c_void_p(sel.ctypes.data),
        C.byref(n_sel), C.c_void_p(sums.ctypes.data) if sums is not None else None)
    return dict(rc=rc, sel=sel[:max(n_sel.value, 0)].copy())


def sync_plan(K, H, gamma, T_c, T_s):
    """Returns (rc, N, h)."""
    N = C.c_int64(0)
    h = C.c_int64(0)
    rc = lib().cocodc_ref_sync_plan(C.c_int32(K), C.c_int32(H), C.c_double(gamma), C.c_double(T_c),
                                    C.c_double(T_s), C.byref(N), C.byref(h))
    return rc, N.value, h.value
