"""Shared helpers of the parity tests: the error metric, the tolerances and adapters that run
the CPU oracle on (sampled rows of) the tensors handed to the HIP library."""
import numpy as np
import torch

from oracle import cref

# Tolerance of the benchmark definition: max abs error relative to the output RMS,
# 1e-5 for the fp32 path and 2e-2 for the bf16 path.  The RMS is taken per query row
# (over heads x features for O, over heads x visible keys for A_n): causal rows average
# very different numbers of values, so their magnitudes differ by an order of magnitude
# and one global RMS would let the small late rows pass with any error at all while the
# bf16 rounding of a single large early-row element already exceeds 2e-2 of it.
TOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").double().numpy()


def n_visible(i, Lq, Lk, causal=True):
    return min(Lk, i + 1 + (Lk - Lq)) if causal else Lk


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max over rows of  max|got - ref| / RMS(ref), rows along axis 0."""
    n = ref.shape[0]
    g, r = got.reshape(n, -1), ref.reshape(n, -1)
    rms = np.sqrt((r * r).mean(axis=1))
    err = np.abs(g - r).max(axis=1)
    assert np.all(rms > 0), "degenerate reference row"
    return float((err / rms).max())


def global_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max|got - ref| over everything / RMS(ref) over everything: the other reading of "relative
    to output RMS".  Logged next to the per-row figure, never asserted (see row_rel_err)."""
    return float(np.abs(got - ref).max() / np.sqrt((ref * ref).mean()))


def bf16_ulps_off(got: np.ndarray, ref: np.ndarray) -> float:
    """For an output that was *stored* as bfloat16: the largest distance, in units of the
    bfloat16 spacing at the reference element, between the stored value and the float64
    reference rounded to bfloat16 (round to nearest even).  A correct float32 result rounded once
    lands on that value or on a neighbour (distance <= 1).  Elements whose spacing is below
    2^-10 of their row's RMS (near-cancellations) are measured in units of that floor instead:
    the float32 accumulation error of a sum does not shrink with the sum."""
    n = ref.shape[0]
    g, r = got.reshape(n, -1), ref.reshape(n, -1)
    rb = torch.from_numpy(r).to(torch.bfloat16).double().numpy()
    with np.errstate(divide="ignore"):
        spacing = np.where(rb != 0, 2.0 ** (np.floor(np.log2(np.abs(rb), where=rb != 0, out=np.zeros_like(rb))) - 7), 0.0)
    rms = np.sqrt((r * r).mean(axis=1, keepdims=True))
    unit = np.maximum(spacing, rms * 2.0 ** -10)
    return float((np.abs(g - rb) / unit).max())


def scores_row_rel_err(got_rows, ref_rows, rows, Lq, Lk, causal=True) -> float:
    """Same metric for score rows [n,H,Lk], restricted to each row's visible keys."""
    worst = 0.0
    for n, i in enumerate(rows):
        nv = n_visible(int(i), Lq, Lk, causal)
        worst = max(worst, row_rel_err(got_rows[n:n + 1, :, :nv], ref_rows[n:n + 1, :, :nv]))
    return worst


def oracle_std_rows(q, k, b, rows, scale=None):
    """Oracle standard scores for batch element b -> [n,H,Lk] float64."""
    return cref.std_scores_rows(f64(q[b]), f64(k[b]), rows, scale)


def oracle_lisa_rows(inp, b, rows, prev_rows, mix=0, delta_scale=None):
    """Oracle LiSA layer for batch element b on the given rows.
    prev_rows: float64 [n,H,Lk].  Returns (A_n rows [n,H,Lk], O rows [n,H,dk])."""
    return cref.lisa_rows(f64(inp["q_lr"][b]), f64(inp["k_lr"][b]), f64(inp["v"][b]),
                          f64(inp["w1"]), f64(inp["w2"]), rows, prev_rows, mix=mix,
                          delta_scale=delta_scale)


def gather_score_rows(scores: torch.Tensor, b: int, rows, Lk=None) -> np.ndarray:
    """scores [B,H,Lq,Lk] (device) -> float64 [n,H,Lk] for batch b, rows.  A 6-dimensional tensor is
    the tiled layout [B,Lq/16,Lk/32,H,16,32]; its rows are cut to Lk keys when Lk is given."""
    idx = torch.as_tensor(np.asarray(rows), device=scores.device, dtype=torch.long)
    if scores.dim() == 6:
        s = scores[b]                                            # [nr, nk, H, 16, 32]
        got = s[idx // 16, :, :, idx % 16, :]                    # [n, nk, H, 32]
        got = got.permute(0, 2, 1, 3)                            # [n, H, nk, 32]
        got = got.reshape(got.shape[0], got.shape[1], -1)
        return f64(got if Lk is None else got[:, :, :Lk])
    return f64(scores[b].index_select(1, idx).permute(1, 0, 2))


def gather_out_rows(out: torch.Tensor, b: int, rows) -> np.ndarray:
    """out [B,Lq,H,dk] -> float64 [n,H,dk]."""
    idx = torch.as_tensor(np.asarray(rows), device=out.device, dtype=torch.long)
    return f64(out[b].index_select(0, idx))


def oracle_project_rows(x, w, b, rows, H, Hkv, r, dk, theta=0.0, pos0=0):
    """Oracle projection front end for batch element b on the given token rows ->
    q [n,H,r], k [n,Hkv,r], v [n,Hkv,dk] float64."""
    return cref.project_rows(f64(x[b]), f64(w), rows, H, Hkv, r, dk, theta=theta or 0.0, pos0=pos0)
