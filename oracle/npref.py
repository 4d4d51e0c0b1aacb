"""Whole-tensor numpy float64 statement of the LiSA layer.  Test infrastructure only.

Written independently of ``lisa_oracle.c``: tensors instead of row loops, ``einsum`` /
``@`` as library steps, masking by -inf instead of a shortened loop.  One sequence per
call; shapes as in the C oracle.  Used on small inputs only (it materialises [H,Lq,Lk]).
"""
import numpy as np

MIX_ADD = 0
MIX_CONCAT = 1


def _expand_kv(x, H):
    """[Hkv, L, c] -> [H, L, c]: query head h uses KV head h // (H // Hkv)."""
    Hkv = x.shape[0]
    return np.repeat(x, H // Hkv, axis=0)


def visible(Lq, Lk):
    """mask[i, j] = True iff key j is visible to query row i (j <= i + Lk - Lq)."""
    i = np.arange(Lq)[:, None]
    j = np.arange(Lk)[None, :]
    return j <= i + (Lk - Lq)


def std_scores(q, k, scale=None):
    """Sec. 2.1 Eq. 2, bracketed term: A = Q K^T / sqrt(d_k), zero where invisible."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    H, Lq, dk = q.shape
    if scale is None:
        scale = 1.0 / np.sqrt(dk)
    a = scale * np.einsum("hid,hjd->hij", q, _expand_kv(k, H))
    return np.where(visible(Lq, k.shape[1])[None], a, 0.0)


def softmax_v(scores, v):
    """Sec. 2.1 Eq. 1-2: P = Softmax(A) over visible keys, O = P V.  Returns (O [Lq,H,dk], P)."""
    scores = np.asarray(scores, np.float64)
    v = np.asarray(v, np.float64)
    H, Lq, Lk = scores.shape
    vis = visible(Lq, Lk)[None]
    a = np.where(vis, scores, -np.inf)
    a = a - a.max(axis=-1, keepdims=True)
    e = np.exp(a)
    p = e / e.sum(axis=-1, keepdims=True)
    o = np.einsum("hij,hjd->ihd", p, _expand_kv(v, H))
    return o, p


def lisa_scores(q_lr, k_lr, w1, w2, prev, mix=MIX_ADD, delta_scale=None):
    """Sec. 5.1 Eq. 3-4: A_n = FFN(A_{n-1}) + A_delta (ADD) or FFN([A_{n-1}; A_delta]) (CONCAT)."""
    q_lr = np.asarray(q_lr, np.float64)
    k_lr = np.asarray(k_lr, np.float64)
    prev = np.asarray(prev, np.float64)
    H, Lq, r = q_lr.shape
    Lk = k_lr.shape[1]
    if delta_scale is None:
        delta_scale = 1.0 / np.sqrt(r)
    a_delta = delta_scale * np.einsum("hit,hjt->hij", q_lr, _expand_kv(k_lr, H))
    at = np.moveaxis(prev, 0, -1)                      # A^T in R^{l x l x h}
    dt = np.moveaxis(a_delta, 0, -1)
    x = np.concatenate([at, dt], axis=-1) if mix == MIX_CONCAT else at
    y = np.maximum(x @ np.asarray(w1, np.float64), 0.0) @ np.asarray(w2, np.float64)
    if mix == MIX_ADD:
        y = y + dt
    a_n = np.moveaxis(y, -1, 0)
    return np.where(visible(Lq, Lk)[None], a_n, 0.0)


def lisa_layer(q_lr, k_lr, v, w1, w2, prev, mix=MIX_ADD, delta_scale=None):
    """Returns (A_n [H,Lq,Lk], O [Lq,H,dk], P [H,Lq,Lk])."""
    a_n = lisa_scores(q_lr, k_lr, w1, w2, prev, mix, delta_scale)
    o, p = softmax_v(a_n, v)
    return a_n, o, p


def huber(a, b, delta=1.0):
    """App. C.1 "Huber loss function": elementwise L_delta(a, b) = (a - b)^2 / 2 where |a - b| <= delta,
    delta (|a - b| - delta / 2) otherwise."""
    d = np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64))
    return np.where(d <= delta, 0.5 * d * d, delta * (d - 0.5 * delta))


def kd_loss(scores, teacher, delta=1.0, causal=True):
    """Sec. 5.1 "Training strategy": the regression term of one LiSA layer, L_delta(A_n, A_n^*), for
    score tensors [..., Lq, Lk]: the mean of the elementwise Huber loss over the entries a query
    row can see (the paper gives no reduction; the mean is the reading taken, that of the usual
    library routine).  L_KD is the mean of this over the layers of S."""
    scores = np.asarray(scores, np.float64)
    teacher = np.asarray(teacher, np.float64)
    Lq, Lk = scores.shape[-2:]
    vis = visible(Lq, Lk) if causal else np.ones((Lq, Lk), bool)
    el = huber(scores, teacher, delta)
    return float(el[..., vis].mean())
