"""Thin ctypes binding of ``liblisa_mi355x.so`` (see include/lisa.h for the contract).

Only argument marshalling happens here: tensors are checked for device, dtype, shape and
contiguity, their device pointers and the current HIP stream are handed to the C ABI, and a
negative status raises ``LisaError``.  There is no fallback: without the built library or
without a GPU the calls fail loudly.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblisa_mi355x.so")

F32, BF16 = 0, 1
MIX_ADD, MIX_CONCAT, MIX_PLUS, MIX_SHARE = 0, 1, 2, 3
ACT_RELU, ACT_SILU, ACT_SINGLE = 0, 1, 2
WS_PREFILL, WS_DECODE, WS_STD, WS_LAYER, WS_LAYER_DECODE, WS_KD = 0, 1, 2, 3, 4, 5

EXPORTS = (
    "lisa_attn_prefill", "lisa_attn_decode", "std_attn_scores", "lisa_workspace_bytes",
    "lisa_scores_bytes", "lisa_score_elem_bytes", "lisa_kcache_saved_bytes", "lisa_supported",
    "lisa_strerror", "lisa_last_hip_error", "lisa_last_path", "lisa_profile_enable",
    "lisa_profile_collect", "lisa_cache_fill", "lisa_project_qkv", "lisa_layer_prefill",
    "lisa_layer_offsets", "lisa_layer_decode", "lisa_tune_set", "lisa_attn_decode_static",
    "lisa_decode_stack", "lisa_stack_workspace_bytes", "lisa_scores_elems", "lisa_kd_huber",
    "lisa_probe_hbm_read", "lisa_probe_hbm_write", "lisa_probe_mfma",
)
TUNE_PREFILL_GROUPS, TUNE_PREFILL_SPLIT, TUNE_PREFILL_PAIR, TUNE_STD_PAIR, TUNE_PROJECT_TN, TUNE_PREFILL_SLICES = range(6)


class LisaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().lisa_strerror(status).decode()
        if status in (-6,):
            msg += ": " + _lib().lisa_last_hip_error().decode()
        super().__init__(f"{where}: {msg} (status {status})")


class Desc(C.Structure):
    _fields_ = [
        ("dtype", C.c_int32), ("B", C.c_int32), ("H", C.c_int32), ("Hkv", C.c_int32),
        ("Lq", C.c_int32), ("Lk", C.c_int32), ("d_k", C.c_int32), ("r", C.c_int32),
        ("F", C.c_int32), ("mix", C.c_int32), ("act", C.c_int32),
        ("delta_scale", C.c_float), ("std_scale", C.c_float), ("causal", C.c_int32),
        ("write_scores", C.c_int32), ("kcache_dim_major", C.c_int32), ("Lmax", C.c_int32),
        ("out_f32", C.c_int32), ("score_tiled", C.c_int32),
    ]


class ProjDesc(C.Structure):
    _fields_ = [
        ("dtype", C.c_int32), ("B", C.c_int32), ("L", C.c_int32), ("d_model", C.c_int32),
        ("H", C.c_int32), ("Hkv", C.c_int32), ("r", C.c_int32), ("d_k", C.c_int32),
        ("Lmax", C.c_int32), ("pos0", C.c_int32), ("kcache_dim_major", C.c_int32),
        ("rope_theta", C.c_float),
    ]


LAYER_STD, LAYER_LISA, LAYER_SHARE = 0, 1, 2


class StackLayer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("reserved", C.c_int32), ("q", C.c_void_p), ("k_cache", C.c_void_p),
                ("v_cache", C.c_void_p), ("w1", C.c_void_p), ("w2", C.c_void_p), ("out", C.c_void_p),
                ("score_row", C.c_void_p)]


class StageTime(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int32), ("total_ms", C.c_float)]


_handle = None


def _lib():
    global _handle
    if _handle is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2408_01890_amd.build` "
                "(there is no CPU fallback)")
        h = C.CDLL(LIB_PATH)
        vp, sz = C.c_void_p, C.c_size_t
        dp = C.POINTER(Desc)
        h.lisa_attn_prefill.argtypes = [dp] + [vp] * 9 + [sz, vp]
        h.lisa_attn_prefill.restype = C.c_int
        h.lisa_attn_decode.argtypes = [dp] + [vp] * 11 + [sz, vp]
        h.lisa_attn_decode.restype = C.c_int
        h.lisa_attn_decode_static.argtypes = [dp] + [vp] * 11
        h.lisa_attn_decode_static.restype = C.c_int
        h.std_attn_scores.argtypes = [dp] + [vp] * 6 + [sz, vp]
        h.std_attn_scores.restype = C.c_int
        h.lisa_workspace_bytes.argtypes = [dp, C.c_int]
        h.lisa_workspace_bytes.restype = sz
        h.lisa_scores_bytes.argtypes = [dp]
        h.lisa_scores_bytes.restype = sz
        h.lisa_scores_elems.argtypes = [dp]
        h.lisa_scores_elems.restype = sz
        h.lisa_kd_huber.argtypes = [dp, vp, vp, C.c_float, C.c_float, C.c_int, vp, vp, sz, vp]
        h.lisa_kd_huber.restype = C.c_int
        h.lisa_score_elem_bytes.argtypes = [dp]
        h.lisa_score_elem_bytes.restype = sz
        h.lisa_kcache_saved_bytes.argtypes = [dp, C.c_int]
        h.lisa_kcache_saved_bytes.restype = sz
        h.lisa_supported.argtypes = [dp]
        h.lisa_supported.restype = C.c_int
        h.lisa_strerror.argtypes = [C.c_int]
        h.lisa_strerror.restype = C.c_char_p
        h.lisa_last_hip_error.restype = C.c_char_p
        h.lisa_last_path.restype = C.c_char_p
        h.lisa_profile_enable.argtypes = [C.c_int]
        h.lisa_profile_enable.restype = C.c_int
        h.lisa_probe_hbm_read.argtypes = [vp, sz, vp, vp]
        h.lisa_probe_hbm_read.restype = C.c_int
        h.lisa_probe_hbm_write.argtypes = [vp, sz, C.c_uint, vp]
        h.lisa_probe_hbm_write.restype = C.c_int
        h.lisa_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_int, vp, vp]
        h.lisa_probe_mfma.restype = C.c_int
        h.lisa_cache_fill.argtypes = [dp] + [vp] * 5
        h.lisa_cache_fill.restype = C.c_int
        h.lisa_project_qkv.argtypes = [C.POINTER(ProjDesc)] + [vp] * 6
        h.lisa_project_qkv.restype = C.c_int
        h.lisa_layer_prefill.argtypes = [dp, C.c_int32, C.c_float] + [vp] * 8 + [sz, vp]
        h.lisa_layer_prefill.restype = C.c_int
        h.lisa_layer_decode.argtypes = [dp, C.c_int32, C.c_float] + [vp] * 10 + [sz, vp]
        h.lisa_layer_decode.restype = C.c_int
        h.lisa_layer_offsets.argtypes = [dp] + [C.POINTER(sz)] * 3
        h.lisa_layer_offsets.restype = C.c_int
        h.lisa_decode_stack.argtypes = [dp, C.POINTER(StackLayer), C.c_int32, vp, sz, vp]
        h.lisa_decode_stack.restype = C.c_int
        h.lisa_stack_workspace_bytes.argtypes = [dp]
        h.lisa_stack_workspace_bytes.restype = sz
        h.lisa_tune_set.argtypes = [C.c_int, C.c_int]
        h.lisa_tune_set.restype = C.c_int
        h.lisa_profile_collect.argtypes = [C.POINTER(StageTime), C.c_int]
        h.lisa_profile_collect.restype = C.c_int
        _handle = h
    return _handle


def library():
    """The loaded ctypes library (raises ImportError if it has not been built)."""
    return _lib()


def make_desc(dtype, B, H, Hkv, Lq, Lk, d_k, r=0, F=0, mix=MIX_ADD, act=ACT_RELU,
              delta_scale=0.0, std_scale=0.0, causal=1, write_scores=0, kcache_dim_major=0,
              Lmax=0, out_f32=0, score_tiled=0) -> Desc:
    code = {torch.float32: F32, torch.bfloat16: BF16, F32: F32, BF16: BF16}[dtype]
    return Desc(code, B, H, Hkv, Lq, Lk, d_k, r, F, mix, act, delta_scale, std_scale, causal,
                write_scores, kcache_dim_major, Lmax, out_f32, score_tiled)


TILE_ROWS, TILE_KEYS = 16, 32


def scores_shape(B, H, Lq, Lk, tiled=False):
    """Shape of a prefill score tensor: [B,H,Lq,Lk], or its tiles [B,ceil(Lq/16),ceil(Lk/32),H,16,32]."""
    if not tiled:
        return (B, H, Lq, Lk)
    return (B, -(-Lq // TILE_ROWS), -(-Lk // TILE_KEYS), H, TILE_ROWS, TILE_KEYS)


def tile_scores(s):
    """[B,H,Lq,Lk] -> tiled layout (a copy; rows and keys padded with zeros to whole tiles)."""
    B, H, Lq, Lk = s.shape
    nr, nk = -(-Lq // TILE_ROWS), -(-Lk // TILE_KEYS)
    p = torch.zeros((B, H, nr * TILE_ROWS, nk * TILE_KEYS), dtype=s.dtype, device=s.device)
    p[:, :, :Lq, :Lk] = s
    return p.view(B, H, nr, TILE_ROWS, nk, TILE_KEYS).permute(0, 2, 4, 1, 3, 5).contiguous()


def untile_scores(t, Lq, Lk):
    """Tiled layout -> [B,H,Lq,Lk] (a copy)."""
    B, nr, nk, H = t.shape[:4]
    return t.permute(0, 3, 1, 4, 2, 5).reshape(B, H, nr * TILE_ROWS, nk * TILE_KEYS)[:, :, :Lq, :Lk].contiguous()


def score_dtype(dtype) -> torch.dtype:
    return torch.float32 if dtype in (torch.float32, F32) else torch.float16


def workspace_bytes(desc: Desc, which: int) -> int:
    return int(_lib().lisa_workspace_bytes(C.byref(desc), which))


def scores_bytes(desc: Desc) -> int:
    return int(_lib().lisa_scores_bytes(C.byref(desc)))


def kcache_saved_bytes(desc: Desc, n_layers: int) -> int:
    return int(_lib().lisa_kcache_saved_bytes(C.byref(desc), n_layers))


def supported(desc: Desc) -> int:
    return int(_lib().lisa_supported(C.byref(desc)))


def last_path() -> str:
    return _lib().lisa_last_path().decode()


class tune:
    """Context manager around lisa_tune_set: forces one kernel geometry (tests), restores the
    library's own choice on exit."""

    def __init__(self, **knobs):
        names = {"prefill_groups": TUNE_PREFILL_GROUPS, "prefill_split": TUNE_PREFILL_SPLIT,
                 "prefill_pair": TUNE_PREFILL_PAIR, "std_pair": TUNE_STD_PAIR, "project_tn": TUNE_PROJECT_TN,
                 "prefill_slices": TUNE_PREFILL_SLICES}
        self.knobs = [(names[k], int(v)) for k, v in knobs.items()]

    def __enter__(self):
        for k, v in self.knobs:
            rc = _lib().lisa_tune_set(k, v)
            if rc:
                raise LisaError(rc, "lisa_tune_set")
        return self

    def __exit__(self, *exc):
        for k, _ in self.knobs:
            _lib().lisa_tune_set(k, -1)
        return False


def probe_hbm_read(buf: torch.Tensor, sink: torch.Tensor) -> None:
    """Reference kernel: one read pass over `buf` (device tensor), nothing written; time it with events."""
    rc = _lib().lisa_probe_hbm_read(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                    C.c_void_p(sink.data_ptr()), _stream())
    if rc:
        raise LisaError(rc, "lisa_probe_hbm_read")


def probe_hbm_write(buf: torch.Tensor, seed: int = 1) -> None:
    """Reference kernel: one write pass over `buf` (device tensor; 16-byte piece i becomes the words
    {seed, i mod 2^32, i / 2^32, ~seed}); time it with events."""
    rc = _lib().lisa_probe_hbm_write(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                     seed & 0xffffffff, _stream())
    if rc:
        raise LisaError(rc, "lisa_probe_hbm_write")


def probe_mfma(shape: int, iters: int, workgroups: int, sink: torch.Tensor) -> None:
    """Reference kernel: `iters` rounds of 2 x 65536 flop of independent MFMAs per wave, four waves per
    workgroup; shape 0 = 16x16x32 f16, 1 = 32x32x16 f16."""
    rc = _lib().lisa_probe_mfma(shape, iters, workgroups, C.c_void_p(sink.data_ptr()), _stream())
    if rc:
        raise LisaError(rc, "lisa_probe_mfma")


def profile_enable(on: bool) -> None:
    _lib().lisa_profile_enable(int(on))


def profile_collect(max_stages: int = 32):
    """{stage name: (launches, total_ms)} of the launches recorded since profile_enable(True)."""
    buf = (StageTime * max_stages)()
    n = _lib().lisa_profile_collect(buf, max_stages)
    if n < 0:
        raise LisaError(n, "lisa_profile_collect")
    return {buf[i].name.decode(): (int(buf[i].launches), float(buf[i].total_ms)) for i in range(n)}


def _ptr(t: Optional[torch.Tensor], name: str, shape=None, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name}: expected a GPU tensor (the library has no CPU path)")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name}: dtype {t.dtype}, expected {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {tuple(t.shape)}, expected {tuple(shape)}")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(nbytes: int, like: torch.Tensor, workspace: Optional[torch.Tensor]):
    if nbytes == 0:
        return workspace, (C.c_void_p(workspace.data_ptr()) if workspace is not None else None), \
            (workspace.numel() * workspace.element_size() if workspace is not None else 0)
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=like.device)
    have = workspace.numel() * workspace.element_size()
    return workspace, C.c_void_p(workspace.data_ptr()), have


def _out_dtype(dt, out_dtype):
    """O is float32 unless the caller asks for the input dtype."""
    out_dtype = torch.float32 if out_dtype is None else out_dtype
    if out_dtype not in (torch.float32, dt):
        raise ValueError(f"out_dtype must be float32 or {dt}")
    return out_dtype, int(out_dtype == torch.float32 and dt != torch.float32)


def std_attn_scores(q, k, v=None, *, want_scores=True, causal=True, std_scale=0.0,
                    scores_out=None, out=None, out_dtype=None, workspace=None, tiled=False):
    """Standard attention that emits the shared scores.  q [B,H,Lq,d_k], k/v [B,Hkv,Lk,d_k].
    Returns (scores [B,H,Lq,Lk] (tiled: see scores_shape) or None, out [B,Lq,H,d_k] or None)."""
    B, H, Lq, dk = q.shape
    _, Hkv, Lk, _ = k.shape
    odt, of32 = _out_dtype(q.dtype, out.dtype if out is not None else out_dtype)
    desc = make_desc(q.dtype, B, H, Hkv, Lq, Lk, dk, causal=int(causal), std_scale=std_scale,
                     out_f32=of32, score_tiled=int(tiled))
    sdt = score_dtype(q.dtype)
    sshape = scores_shape(B, H, Lq, Lk, tiled)
    if want_scores and scores_out is None:
        scores_out = torch.empty(sshape, dtype=sdt, device=q.device)
    if v is not None and out is None:
        out = torch.empty((B, Lq, H, dk), dtype=odt, device=q.device)
    need = workspace_bytes(desc, WS_STD) if out is not None else 0
    workspace, wp, wb = _workspace(need, q, workspace)
    rc = _lib().std_attn_scores(
        C.byref(desc), _ptr(q, "q", dtype=q.dtype), _ptr(k, "k", (B, Hkv, Lk, dk), q.dtype),
        _ptr(v, "v", (B, Hkv, Lk, dk), q.dtype), _ptr(scores_out, "scores_out", sshape, sdt),
        _ptr(out, "out", (B, Lq, H, dk), odt), wp, wb, _stream())
    if rc:
        raise LisaError(rc, "std_attn_scores")
    return scores_out, out


def std_attn_decode(q, k_cache, v_cache, Lk, *, want_scores=True, std_scale=0.0,
                    score_row_out=None, out=None, out_dtype=None, workspace=None):
    """Decode step of a standard layer: q [B,H,d_k] against caches [B,Hkv,Lmax,d_k], first Lk
    keys.  Returns (score row [B,H,Lk] or None, out [B,H,d_k])."""
    B, H, dk = q.shape
    _, Hkv, Lmax, _ = k_cache.shape
    odt, of32 = _out_dtype(q.dtype, out.dtype if out is not None else out_dtype)
    desc = make_desc(q.dtype, B, H, Hkv, 1, Lk, dk, std_scale=std_scale, Lmax=Lmax, out_f32=of32)
    sdt = score_dtype(q.dtype)
    if want_scores and score_row_out is None:
        score_row_out = torch.empty((B, H, Lk), dtype=sdt, device=q.device)
    if out is None:
        out = torch.empty((B, H, dk), dtype=odt, device=q.device)
    need = workspace_bytes(desc, WS_STD)
    workspace, wp, wb = _workspace(need, q, workspace)
    rc = _lib().std_attn_scores(
        C.byref(desc), _ptr(q, "q", dtype=q.dtype), _ptr(k_cache, "k_cache", dtype=q.dtype),
        _ptr(v_cache, "v_cache", (B, Hkv, Lmax, dk), q.dtype),
        _ptr(score_row_out, "score_row_out", (B, H, Lk), sdt), _ptr(out, "out", (B, H, dk), odt),
        wp, wb, _stream())
    if rc:
        raise LisaError(rc, "std_attn_scores(decode)")
    return score_row_out, out


def lisa_attn_prefill(q_lr, k_lr, v, scores_prev, w1, w2, *, mix=MIX_ADD, act=ACT_RELU,
                      write_scores=True, causal=True, delta_scale=0.0, out=None, out_dtype=None,
                      scores_out=None, workspace=None, tiled=False, Lq=None):
    """One LiSA layer.  q_lr [B,H,Lq,r], k_lr [B,Hkv,Lk,r], v [B,Hkv,Lk,d_k],
    scores_prev [B,H,Lq,Lk] (score dtype), w1 [Din,F], w2 [F,H].  Operands a variant does not
    use are None: w1, w2 for MIX_PLUS / MIX_SHARE, w2 for ACT_SINGLE, q_lr, k_lr for MIX_SHARE.
    tiled: both score tensors are in the tiled layout (see scores_shape); Lq is then taken from
    q_lr (or the Lq argument where there is no q_lr).
    Returns (out [B,Lq,H,d_k], scores_out [B,H,Lq,Lk] or None)."""
    if tiled:
        B, H = scores_prev.shape[0], scores_prev.shape[3]
        Lq = q_lr.shape[2] if q_lr is not None else Lq
        Lk = v.shape[2]
    else:
        B, H, Lq, Lk = scores_prev.shape
    sshape = scores_shape(B, H, Lq, Lk, tiled)
    _, Hkv, _, dk = v.shape
    r = q_lr.shape[3] if q_lr is not None else 0
    has_ffn = mix in (MIX_ADD, MIX_CONCAT)
    Din, F = w1.shape if has_ffn else (0, 0)
    dt = v.dtype
    sdt = score_dtype(dt)
    odt, of32 = _out_dtype(dt, out.dtype if out is not None else out_dtype)
    desc = make_desc(dt, B, H, Hkv, Lq, Lk, dk, r, F, mix=mix, act=act, delta_scale=delta_scale,
                     causal=int(causal), write_scores=int(write_scores), out_f32=of32,
                     score_tiled=int(tiled))
    if has_ffn and Din != (2 * H if mix == MIX_CONCAT else H):
        raise ValueError(f"w1 has {Din} rows, expected {2 * H if mix == MIX_CONCAT else H}")
    if out is None:
        out = torch.empty((B, Lq, H, dk), dtype=odt, device=v.device)
    if write_scores and scores_out is None:
        scores_out = torch.empty(sshape, dtype=sdt, device=v.device)
    need = workspace_bytes(desc, WS_PREFILL)
    if need == 0 and supported(desc) != 0:
        raise LisaError(supported(desc), "lisa_attn_prefill")
    workspace, wp, wb = _workspace(need, v, workspace)
    rc = _lib().lisa_attn_prefill(
        C.byref(desc), _ptr(q_lr, "q_lr", (B, H, Lq, r), dt), _ptr(k_lr, "k_lr", (B, Hkv, Lk, r), dt),
        _ptr(v, "v", (B, Hkv, Lk, dk), dt), _ptr(scores_prev, "scores_prev", sshape, sdt),
        _ptr(w1 if has_ffn else None, "w1", (Din, F), dt),
        _ptr(w2 if has_ffn and act != ACT_SINGLE else None, "w2", (F, H), dt),
        _ptr(out, "out", (B, Lq, H, dk), odt),
        _ptr(scores_out if write_scores else None, "scores_out", sshape, sdt), wp, wb,
        _stream())
    if rc:
        raise LisaError(rc, "lisa_attn_prefill")
    return out, (scores_out if write_scores else None)


def lisa_kd_huber(scores, teacher, *, Lq=None, Lk=None, delta=1.0, weight=1.0, accumulate=False, causal=True,
                  tiled=False, out=None, workspace=None):
    """Huber regression term of the distillation loss for one layer (see include/lisa.h): mean over
    the visible entries of L_delta(scores, teacher).  scores, teacher: [B,H,Lq,Lk], or tiled (then
    Lq and Lk are given).  Returns the device tensor out (2 float64: accumulated loss, this mean)."""
    if tiled:
        B, H = scores.shape[0], scores.shape[3]
    else:
        B, H, Lq, Lk = scores.shape
    dt = torch.float32 if scores.dtype == torch.float32 else torch.bfloat16
    desc = make_desc(dt, B, H, H, Lq, Lk, 1, causal=int(causal), score_tiled=int(tiled))
    sshape = scores_shape(B, H, Lq, Lk, tiled)
    if out is None:
        out = torch.zeros(2, dtype=torch.float64, device=scores.device)
    need = workspace_bytes(desc, WS_KD)
    workspace, wp, wb = _workspace(need, scores, workspace)
    rc = _lib().lisa_kd_huber(C.byref(desc), _ptr(scores, "scores", sshape, scores.dtype),
                              _ptr(teacher, "teacher", sshape, scores.dtype), float(delta), float(weight),
                              int(bool(accumulate)), _ptr(out, "out", (2,), torch.float64), wp, wb, _stream())
    if rc:
        raise LisaError(rc, "lisa_kd_huber")
    return out


def lisa_cache_fill(k_lr, v, k_lr_cache, v_cache, *, dim_major=True):
    """Prefill -> decode hand-over: copies k_lr [B,Hkv,Lk,r] and v [B,Hkv,Lk,d_k] into the first
    Lk key slots of k_lr_cache ([B,Hkv,r,Lmax] if dim_major else [B,Hkv,Lmax,r]) and
    v_cache [B,Hkv,Lmax,d_k]."""
    B, Hkv, Lk, r = k_lr.shape
    _, _, Lmax, dk = v_cache.shape
    dt = k_lr.dtype
    desc = make_desc(dt, B, Hkv, Hkv, 1, Lk, dk, r, kcache_dim_major=int(dim_major), Lmax=Lmax)
    kshape = (B, Hkv, r, Lmax) if dim_major else (B, Hkv, Lmax, r)
    rc = _lib().lisa_cache_fill(
        C.byref(desc), _ptr(k_lr, "k_lr", dtype=dt), _ptr(v, "v", (B, Hkv, Lk, dk), dt),
        _ptr(k_lr_cache, "k_lr_cache", kshape, dt), _ptr(v_cache, "v_cache", (B, Hkv, Lmax, dk), dt),
        _stream())
    if rc:
        raise LisaError(rc, "lisa_cache_fill")
    return k_lr_cache, v_cache


def lisa_project_qkv(x, w, H, Hkv, r, d_k, *, rope_theta=0.0, pos0=0, q_lr=None, k_lr=None, v=None,
                     dim_major=False):
    """Front end of a LiSA layer: x [B,L,d] times the stacked weight rows w [H*r + Hkv*r + Hkv*d_k, d]
    (W^Q_LR, W^K_LR, W^V, one row per output feature), rotary embedding on Q_LR / K_LR when
    rope_theta > 0.  Writes q_lr [B,H,L,r] and, at key indices pos0 .. pos0+L-1, k_lr
    ([B,Hkv,r,Lmax] if dim_major else [B,Hkv,Lmax,r]) and v [B,Hkv,Lmax,d_k]; tensors that are
    not passed are allocated dense (Lmax = pos0 + L).  Returns (q_lr, k_lr, v)."""
    B, L, D = x.shape
    dt = x.dtype
    dev = x.device
    Lmax = v.shape[2] if v is not None else pos0 + L
    kshape = (B, Hkv, r, Lmax) if dim_major else (B, Hkv, Lmax, r)
    if q_lr is None:
        q_lr = torch.empty((B, H, L, r), dtype=dt, device=dev)
    if k_lr is None:
        k_lr = torch.empty(kshape, dtype=dt, device=dev)
    if v is None:
        v = torch.empty((B, Hkv, Lmax, d_k), dtype=dt, device=dev)
    code = {torch.float32: F32, torch.bfloat16: BF16}[dt]
    desc = ProjDesc(code, B, L, D, H, Hkv, r, d_k, Lmax, pos0, int(dim_major), float(rope_theta or 0.0))
    rc = _lib().lisa_project_qkv(
        C.byref(desc), _ptr(x, "x", dtype=dt), _ptr(w, "w", ((H + Hkv) * r + Hkv * d_k, D), dt),
        _ptr(q_lr, "q_lr", (B, H, L, r), dt), _ptr(k_lr, "k_lr", kshape, dt),
        _ptr(v, "v", (B, Hkv, Lmax, d_k), dt), _stream())
    if rc:
        raise LisaError(rc, "lisa_project_qkv")
    return q_lr, k_lr, v


def lisa_layer_prefill(x, w_qkv, Hkv, r, d_k, scores_prev, w1, w2, *, rope_theta=0.0, mix=MIX_ADD,
                       write_scores=True, causal=True, out=None, out_dtype=None, scores_out=None,
                       workspace=None, tiled=False):
    """A whole LiSA layer from the hidden states x [B,L,d]: projection front end (see
    lisa_project_qkv) then lisa_attn_prefill.  Returns (out, scores_out or None, (q_lr, k_lr, v)),
    the last being views of the workspace."""
    B, L, D = x.shape
    H = scores_prev.shape[3] if tiled else scores_prev.shape[1]
    Din, F = w1.shape
    dt = x.dtype
    sdt = score_dtype(dt)
    odt, of32 = _out_dtype(dt, out.dtype if out is not None else out_dtype)
    desc = make_desc(dt, B, H, Hkv, L, L, d_k, r, F, mix=mix, causal=int(causal),
                     write_scores=int(write_scores), out_f32=of32, score_tiled=int(tiled))
    sshape = scores_shape(B, H, L, L, tiled)
    if out is None:
        out = torch.empty((B, L, H, d_k), dtype=odt, device=x.device)
    if write_scores and scores_out is None:
        scores_out = torch.empty(sshape, dtype=sdt, device=x.device)
    need = workspace_bytes(desc, WS_LAYER)
    if need == 0:
        raise LisaError(supported(desc) or -2, "lisa_layer_prefill")
    workspace, wp, wb = _workspace(need, x, workspace)
    rc = _lib().lisa_layer_prefill(
        C.byref(desc), D, float(rope_theta or 0.0), _ptr(x, "x", dtype=dt),
        _ptr(w_qkv, "w_qkv", ((H + Hkv) * r + Hkv * d_k, D), dt),
        _ptr(scores_prev, "scores_prev", sshape, sdt), _ptr(w1, "w1", dtype=dt),
        _ptr(w2, "w2", (F, H), dt), _ptr(out, "out", (B, L, H, d_k), odt),
        _ptr(scores_out if write_scores else None, "scores_out", sshape, sdt), wp, wb, _stream())
    if rc:
        raise LisaError(rc, "lisa_layer_prefill")
    offs = [C.c_size_t() for _ in range(3)]
    _lib().lisa_layer_offsets(C.byref(desc), *[C.byref(o) for o in offs])
    es = x.element_size()

    def view(off, shape):
        n = 1
        for d in shape:
            n *= d
        return workspace[off.value:off.value + n * es].view(dt).view(shape)

    qkv = (view(offs[0], (B, H, L, r)), view(offs[1], (B, Hkv, L, r)), view(offs[2], (B, Hkv, L, d_k)))
    return out, (scores_out if write_scores else None), qkv


def lisa_layer_decode(x, w_qkv, k_lr_cache, v_cache, Lk, score_row_prev, w1, w2, *, rope_theta=0.0,
                      dim_major=True, mix=MIX_ADD, act=ACT_RELU, write_scores=True, out=None,
                      out_dtype=None, score_row_out=None, workspace=None):
    """Decode step of a whole LiSA layer from the hidden states x [B,d] of the new tokens (position
    Lk-1): projection straight into the caches, then lisa_attn_decode.
    Returns (out [B,H,d_k], score_row_out [B,H,Lk] or None)."""
    B, D = x.shape
    _, H, _ = score_row_prev.shape
    _, Hkv, Lmax, dk = v_cache.shape
    r = k_lr_cache.shape[2] if dim_major else k_lr_cache.shape[3]
    has_ffn = mix in (MIX_ADD, MIX_CONCAT)
    Din, F = w1.shape if has_ffn else (0, 0)
    if not has_ffn:
        w1 = w2 = None
    elif act == ACT_SINGLE:
        w2 = None
    dt = x.dtype
    sdt = score_dtype(dt)
    odt, of32 = _out_dtype(dt, out.dtype if out is not None else out_dtype)
    desc = make_desc(dt, B, H, Hkv, 1, Lk, dk, r, F, mix=mix, act=act, write_scores=int(write_scores),
                     kcache_dim_major=int(dim_major), Lmax=Lmax, out_f32=of32)
    kshape = (B, Hkv, r, Lmax) if dim_major else (B, Hkv, Lmax, r)
    if out is None:
        out = torch.empty((B, H, dk), dtype=odt, device=x.device)
    if write_scores and score_row_out is None:
        score_row_out = torch.empty((B, H, Lk), dtype=sdt, device=x.device)
    need = workspace_bytes(desc, WS_LAYER_DECODE)
    if need == 0:
        raise LisaError(supported(desc) or -2, "lisa_layer_decode")
    workspace, wp, wb = _workspace(need, x, workspace)
    rc = _lib().lisa_layer_decode(
        C.byref(desc), D, float(rope_theta or 0.0), _ptr(x, "x", dtype=dt),
        _ptr(w_qkv, "w_qkv", ((H + Hkv) * r + Hkv * dk, D), dt), _ptr(k_lr_cache, "k_lr_cache", kshape, dt),
        _ptr(v_cache, "v_cache", dtype=dt), _ptr(score_row_prev, "score_row_prev", (B, H, Lk), sdt),
        _ptr(w1, "w1", (Din, F), dt), _ptr(w2, "w2", (F, H), dt), _ptr(out, "out", (B, H, dk), odt),
        _ptr(score_row_out if write_scores else None, "score_row_out", (B, H, Lk), sdt), wp, wb, _stream())
    if rc:
        raise LisaError(rc, "lisa_layer_decode")
    return out, (score_row_out if write_scores else None)


def lisa_attn_decode(q_lr, k_lr_cache, v_cache, Lk, score_row_prev, w1, w2, *, k_lr_new=None,
                     v_new=None, dim_major=True, mix=MIX_ADD, act=ACT_RELU, write_scores=True,
                     delta_scale=0.0, out=None, out_dtype=None, score_row_out=None, workspace=None,
                     static_scratch=False):
    """One LiSA decode step.  q_lr [B,H,r]; k_lr_cache [B,Hkv,r,Lmax] (dim_major) or
    [B,Hkv,Lmax,r]; v_cache [B,Hkv,Lmax,d_k]; score_row_prev [B,H,Lk].
    static_scratch: call lisa_attn_decode_static (no workspace; pass `out` and `score_row_out`
    if the call itself must not allocate).
    Returns (out [B,H,d_k], score_row_out [B,H,Lk] or None)."""
    B, H, _ = score_row_prev.shape
    r = q_lr.shape[2] if q_lr is not None else 0
    _, Hkv, Lmax, dk = v_cache.shape
    has_ffn = mix in (MIX_ADD, MIX_CONCAT)
    Din, F = w1.shape if has_ffn else (0, 0)
    if not has_ffn:
        w1 = w2 = None
    elif act == ACT_SINGLE:
        w2 = None
    dt = v_cache.dtype
    sdt = score_dtype(dt)
    odt, of32 = _out_dtype(dt, out.dtype if out is not None else out_dtype)
    desc = make_desc(dt, B, H, Hkv, 1, Lk, dk, r, F, mix=mix, act=act, delta_scale=delta_scale,
                     write_scores=int(write_scores), kcache_dim_major=int(dim_major), Lmax=Lmax,
                     out_f32=of32)
    kshape = (B, Hkv, r, Lmax) if dim_major else (B, Hkv, Lmax, r)
    if out is None:
        out = torch.empty((B, H, dk), dtype=odt, device=v_cache.device)
    if write_scores and score_row_out is None:
        score_row_out = torch.empty((B, H, Lk), dtype=sdt, device=v_cache.device)
    args = [C.byref(desc), _ptr(q_lr, "q_lr", dtype=dt), _ptr(k_lr_new, "k_lr_new", (B, Hkv, r), dt),
            _ptr(v_new, "v_new", (B, Hkv, dk), dt), _ptr(k_lr_cache, "k_lr_cache", kshape, dt),
            _ptr(v_cache, "v_cache", dtype=dt), _ptr(score_row_prev, "score_row_prev", (B, H, Lk), sdt),
            _ptr(w1, "w1", (Din, F), dt), _ptr(w2, "w2", (F, H), dt), _ptr(out, "out", (B, H, dk), odt),
            _ptr(score_row_out if write_scores else None, "score_row_out", (B, H, Lk), sdt)]
    if static_scratch:
        rc = _lib().lisa_attn_decode_static(*args, _stream())
    else:
        need = workspace_bytes(desc, WS_DECODE)
        workspace, wp, wb = _workspace(need, v_cache, workspace)
        rc = _lib().lisa_attn_decode(*args, wp, wb, _stream())
    if rc:
        raise LisaError(rc, "lisa_attn_decode_static" if static_scratch else "lisa_attn_decode")
    return out, (score_row_out if write_scores else None)


def stack_workspace_bytes(desc: Desc) -> int:
    return int(_lib().lisa_stack_workspace_bytes(C.byref(desc)))


class DecodeStack:
    """Marshals one decode step through a stack of attention layers (lisa_decode_stack).

    `layers`: list of dicts with key "kind" (LAYER_STD | LAYER_LISA | LAYER_SHARE) and tensors
    "q" (STD: q [B,H,d_k]; LISA: q_lr [B,H,r]), "k_cache" (STD: K cache; LISA: K_LR cache),
    "v_cache" [B,Hkv,Lmax,d_k], "w1", "w2" (LISA), optional "out" [B,H,d_k] float32 and
    "score_row" [B,H,Lk].  The array of layer records is built once; step() only makes the call."""

    def __init__(self, layers, Lk, *, r, F, dim_major=True, mix=MIX_ADD, act=ACT_RELU, keep_rows=False):
        v0 = layers[0]["v_cache"]
        B, Hkv, Lmax, dk = v0.shape
        H = layers[0]["q"].shape[1]
        dt = v0.dtype
        self.sdt = score_dtype(dt)
        self.desc = make_desc(dt, B, H, Hkv, 1, Lk, dk, r, F, mix=mix, act=act, kcache_dim_major=int(dim_major),
                              Lmax=Lmax, out_f32=1)
        self.outs, self.rows, self._keep = [], [], []
        arr = (StackLayer * len(layers))()
        for n, ly in enumerate(layers):
            out = ly.get("out")
            if out is None:
                out = torch.empty((B, H, dk), dtype=torch.float32, device=v0.device)
            row = ly.get("score_row")
            if row is None and keep_rows:
                row = torch.empty((B, H, Lk), dtype=self.sdt, device=v0.device)
            kind = ly["kind"]
            kshape = None
            if kind == LAYER_STD:
                kshape = (B, Hkv, Lmax, dk)
            elif kind == LAYER_LISA:
                kshape = (B, Hkv, r, Lmax) if dim_major else (B, Hkv, Lmax, r)
            share = kind == LAYER_SHARE
            arr[n] = StackLayer(
                kind, 0,
                None if share else _ptr(ly["q"], "q", (B, H, dk if kind == LAYER_STD else r), dt),
                None if share else _ptr(ly["k_cache"], "k_cache", kshape, dt),
                _ptr(ly["v_cache"], "v_cache", (B, Hkv, Lmax, dk), dt),
                _ptr(ly.get("w1"), "w1", dtype=dt) if kind == LAYER_LISA else None,
                _ptr(ly.get("w2"), "w2", dtype=dt) if kind == LAYER_LISA else None,
                _ptr(out, "out", (B, H, dk), torch.float32),
                _ptr(row, "score_row", (B, H, Lk), self.sdt))
            self.outs.append(out)
            self.rows.append(row)
            self._keep.append(ly)
        self.arr = arr
        need = stack_workspace_bytes(self.desc)
        if need == 0:
            raise LisaError(supported(self.desc) or -2, "lisa_decode_stack")
        self.ws = torch.empty(need, dtype=torch.uint8, device=v0.device)

    def step(self):
        rc = _lib().lisa_decode_stack(C.byref(self.desc), self.arr, len(self.arr), C.c_void_p(self.ws.data_ptr()),
                                      self.ws.numel(), _stream())
        if rc:
            raise LisaError(rc, "lisa_decode_stack")
        return self.outs
