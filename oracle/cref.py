"""ctypes binding of the C oracle (``lisa_oracle.c``).  Test infrastructure only.

All arrays are float64, C-contiguous, one sequence per call (see the C header comment
for the layouts).  Functions return freshly allocated numpy arrays.
"""
import ctypes as C

import numpy as np

from . import build as _build

MIX_ADD = 0
MIX_CONCAT = 1
MIX_PLUS = 2
MIX_SHARE = 3
ACT_RELU = 0
ACT_SILU = 1
ACT_SINGLE = 2

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.lisa_oracle_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().lisa_oracle_num_threads())


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _rows(rows):
    r = np.ascontiguousarray(rows, dtype=np.int32)
    return r, r.ctypes.data_as(C.POINTER(C.c_int))


def std_scores_rows(q, k, rows, scale=None):
    """A[h,i,j] = scale <q[h,i], k[kv(h),j]> for the requested rows -> [n_rows, H, Lk]."""
    q, qp = _d(q)
    k, kp = _d(k)
    H, Lq, dk = q.shape
    Hkv, Lk, dk2 = k.shape
    assert dk == dk2
    if scale is None:
        scale = 1.0 / np.sqrt(dk)
    rows, rp = _rows(rows)
    out = np.empty((len(rows), H, Lk), dtype=np.float64)
    rc = lib().lisa_oracle_std_scores_rows(H, Hkv, Lq, Lk, dk, C.c_double(scale), qp, kp,
                                           len(rows), rp, out.ctypes.data_as(C.POINTER(C.c_double)))
    if rc:
        raise ValueError("lisa_oracle_std_scores_rows: bad shape")
    return out


def softmax_v_rows(v, rows, scores_rows, Lq, want_probs=False):
    """Causal softmax of the given score rows times V -> out [n_rows, H, dk] (and P)."""
    v, vp = _d(v)
    s, sp = _d(scores_rows)
    Hkv, Lk, dk = v.shape
    n, H, Lk2 = s.shape
    assert Lk == Lk2
    rows, rp = _rows(rows)
    assert len(rows) == n
    out = np.empty((n, H, dk), dtype=np.float64)
    probs = np.empty((n, H, Lk), dtype=np.float64) if want_probs else None
    pp = probs.ctypes.data_as(C.POINTER(C.c_double)) if want_probs else None
    rc = lib().lisa_oracle_softmax_v_rows(H, Hkv, Lq, Lk, dk, vp, n, rp, sp, pp,
                                          out.ctypes.data_as(C.POINTER(C.c_double)))
    if rc:
        raise ValueError("lisa_oracle_softmax_v_rows: bad shape")
    return (out, probs) if want_probs else out


def lisa_rows(q_lr, k_lr, v, w1, w2, rows, prev_rows, mix=MIX_ADD, delta_scale=None,
              want_probs=False, act=ACT_RELU, Lq=None):
    """One LiSA layer for the requested query rows.

    Returns (scores [n,H,Lk], out [n,H,dk]) and P [n,H,Lk] when ``want_probs``.
    ``w1`` / ``w2`` may be None for the variants without an FFN (MIX_PLUS, MIX_SHARE), ``w2``
    for ACT_SINGLE, ``q_lr`` / ``k_lr`` for MIX_SHARE (then pass ``Lq``).
    """
    v, vp = _d(v)
    prev, pp = _d(prev_rows)
    Hkv, Lk, dk = v.shape
    rows, rp = _rows(rows)
    n = len(rows)
    H = prev.shape[1]
    assert prev.shape == (n, H, Lk)
    has_ffn = mix in (MIX_ADD, MIX_CONCAT)
    null = C.POINTER(C.c_double)()
    if q_lr is not None:
        q_lr, qp = _d(q_lr)
        k_lr, kp = _d(k_lr)
        assert q_lr.shape[0] == H and k_lr.shape[:2] == (Hkv, Lk) and q_lr.shape[2] == k_lr.shape[2]
        Lq, r = q_lr.shape[1], q_lr.shape[2]
    else:
        assert mix == MIX_SHARE and Lq is not None
        qp = kp = null
        r = 0
    F = 0
    w1p = w2p = null
    if has_ffn:
        w1, w1p = _d(w1)
        Din, F = w1.shape
        assert Din == (2 * H if mix == MIX_CONCAT else H)
        if act != ACT_SINGLE:
            w2, w2p = _d(w2)
            assert w2.shape == (F, H)
    if delta_scale is None:
        delta_scale = 1.0 / np.sqrt(r) if r > 0 else 0.0
    scores = np.empty((n, H, Lk), dtype=np.float64)
    out = np.empty((n, H, dk), dtype=np.float64)
    probs = np.empty((n, H, Lk), dtype=np.float64) if want_probs else None
    prp = probs.ctypes.data_as(C.POINTER(C.c_double)) if want_probs else None
    rc = lib().lisa_oracle_lisa_rows(H, Hkv, Lq, Lk, dk, r, F, int(mix), int(act),
                                     C.c_double(delta_scale), qp, kp, vp, w1p, w2p, n, rp, pp,
                                     scores.ctypes.data_as(C.POINTER(C.c_double)), prp,
                                     out.ctypes.data_as(C.POINTER(C.c_double)))
    if rc:
        raise ValueError("lisa_oracle_lisa_rows: bad shape")
    return (scores, out, probs) if want_probs else (scores, out)


def project_rows(x, w, rows, H, Hkv, r, dk, theta=0.0, pos0=0):
    """Projection front end for the requested token rows of one sequence.

    x [L,D], w [H*r + Hkv*r + Hkv*dk, D] -> q [n,H,r], k [n,Hkv,r], v [n,Hkv,dk]
    (rotary embedding on q, k when theta > 0).
    """
    x, xp = _d(x)
    w, wp = _d(w)
    L, D = x.shape
    assert w.shape == (H * r + Hkv * r + Hkv * dk, D)
    rows, rp = _rows(rows)
    n = len(rows)
    q = np.empty((n, H, r), dtype=np.float64)
    k = np.empty((n, Hkv, r), dtype=np.float64)
    v = np.empty((n, Hkv, dk), dtype=np.float64)
    dp = C.POINTER(C.c_double)
    rc = lib().lisa_oracle_project_rows(L, D, H, Hkv, r, dk, C.c_double(theta), int(pos0), xp, wp,
                                        n, rp, q.ctypes.data_as(dp), k.ctypes.data_as(dp),
                                        v.ctypes.data_as(dp))
    if rc:
        raise ValueError("lisa_oracle_project_rows: bad shape")
    return q, k, v
