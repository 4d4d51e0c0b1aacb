"""Pins of the float64 oracle against things other than itself (CPU only).

Each test fixes one part of the oracle to what the paper or the mathematics determine:
hand-evaluated numbers, closed forms, brute force in pure Python, library softmax/matmul,
and the worked head-permutation example of Sec. 5.1.  A dropped term, a wrong sign or
index, or a transposed operand in the oracle fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import cref, npref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def all_rows(L):
    return np.arange(L, dtype=np.int32)


def identity_ffn(H, F):
    """[I,-I] then [I;-I]: relu(x) - relu(-x) = x exactly."""
    w1 = np.zeros((H, F))
    w2 = np.zeros((F, H))
    w1[:, :H] = np.eye(H)
    w1[:, H:2 * H] = -np.eye(H)
    w2[:H] = np.eye(H)
    w2[H:2 * H] = -np.eye(H)
    return w1, w2


# --------------------------------------------------------------------------------------
# 1. A hand-evaluated two-head example (every number below was worked out on paper).
# --------------------------------------------------------------------------------------
HAND = dict(
    q_lr=np.array([[[1.0], [2.0], [-1.0]], [[0.5], [-1.0], [2.0]]]),        # [H=2, L=3, r=1]
    k_lr=np.array([[[2.0], [-1.0], [1.0]], [[1.0], [1.0], [-2.0]]]),
    v=np.array([[[1.0, 0.0], [0.0, 1.0], [2.0, 2.0]], [[1.0, 1.0], [-1.0, 0.0], [0.0, 3.0]]]),
    w1=np.array([[1.0, -1.0, 0.0, 2.0], [0.0, 1.0, -1.0, 1.0]]),            # [2, 4]
    w2=np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0], [0.5, -1.0]]),         # [4, 2]
    prev=np.array([[[3.0, 9.0, 9.0], [2.0, -1.0, 9.0], [1.0, 0.0, -1.0]],   # [H, L, L]; the 9s
                   [[-2.0, 9.0, 9.0], [1.0, 1.0, 9.0], [0.0, 2.0, 1.0]]]),  # are above the diagonal
)
# A_n (ADD, delta_scale = 1) by hand:
#  (0,0): x=[3,-2] -> W1^T x=[3,-5,2,4] -> relu [3,0,2,4] -> y=[3+2+2, 2-4]=[7,-2]; a_delta=[2,0.5] -> [9,-1.5]
#  (1,0): x=[2,1] -> [2,-1,-1,5] -> [2,0,0,5] -> y=[4.5,-5]; a_delta=[4,-1] -> [8.5,-6]
#  (1,1): x=[-1,1] -> [-1,2,-1,-1] -> [0,2,0,0] -> y=[0,2]; a_delta=[-2,-1] -> [-2,1]
#  (2,0): x=[1,0] -> [1,-1,0,2] -> [1,0,0,2] -> y=[2,-2]; a_delta=[-2,2] -> [0,0]
#  (2,1): x=[0,2] -> [0,2,-2,2] -> [0,2,0,2] -> y=[1,0]; a_delta=[1,2] -> [2,2]
#  (2,2): x=[-1,1] -> y=[0,2]; a_delta=[-1,-4] -> [-1,-2]
HAND_AN = np.array([[[9.0, 0, 0], [8.5, -2.0, 0], [0.0, 2.0, -1.0]],
                    [[-1.5, 0, 0], [-6.0, 1.0, 0], [0.0, 2.0, -2.0]]])


def hand_out():
    e = math.exp
    o = np.zeros((3, 2, 2))
    o[0, 0] = [1.0, 0.0]
    o[0, 1] = [1.0, 1.0]
    # row 1, head 0: scores [8.5,-2] -> weights 1, e^-10.5
    z = 1.0 + e(-10.5)
    o[1, 0] = [1.0 / z, e(-10.5) / z]
    # row 1, head 1: scores [-6, 1] -> weights e^-7, 1
    z = e(-7.0) + 1.0
    o[1, 1] = [(e(-7.0) - 1.0) / z, e(-7.0) / z]
    # row 2, head 0: scores [0,2,-1] -> weights e^-2, 1, e^-3 on V rows [1,0],[0,1],[2,2]
    z = e(-2.0) + 1.0 + e(-3.0)
    o[2, 0] = [(e(-2.0) + 2 * e(-3.0)) / z, (1.0 + 2 * e(-3.0)) / z]
    # row 2, head 1: scores [0,2,-2] -> weights e^-2, 1, e^-4 on V rows [1,1],[-1,0],[0,3]
    z = e(-2.0) + 1.0 + e(-4.0)
    o[2, 1] = [(e(-2.0) - 1.0) / z, (e(-2.0) + 3 * e(-4.0)) / z]
    return o


@pytest.mark.parametrize("impl", ["c", "numpy"])
def test_hand_example_add(impl):
    d = HAND
    if impl == "c":
        prev_rows = np.ascontiguousarray(np.transpose(d["prev"], (1, 0, 2)))
        a_n, out = cref.lisa_rows(d["q_lr"], d["k_lr"], d["v"], d["w1"], d["w2"], all_rows(3),
                                  prev_rows, mix=cref.MIX_ADD, delta_scale=1.0)
        a_n = np.transpose(a_n, (1, 0, 2))
    else:
        a_n, out, _ = npref.lisa_layer(d["q_lr"], d["k_lr"], d["v"], d["w1"], d["w2"], d["prev"],
                                       mix=npref.MIX_ADD, delta_scale=1.0)
    np.testing.assert_allclose(a_n, HAND_AN, rtol=0, atol=1e-14)
    np.testing.assert_allclose(out, hand_out(), rtol=0, atol=1e-14)


@pytest.mark.parametrize("impl", ["c", "numpy"])
def test_hand_example_concat_position(impl):
    """One position by hand in CONCAT mode: x = [A_prev ; a_delta] = [1, 0, -2, 2] at (2,0).
    W1 rows for A_prev as above, rows for a_delta = [[0,1,0,0],[1,0,0,-1]]:
    W1^T x = [1+2, -1-2, 0, 2-2] = [3,-3,0,0] -> relu [3,0,0,0] -> y = [3, 0] = A_n (no addition)."""
    d = HAND
    w1c = np.vstack([d["w1"], np.array([[0.0, 1.0, 0.0, 0.0], [1.0, 0.0, 0.0, -1.0]])])
    if impl == "c":
        prev_rows = np.ascontiguousarray(np.transpose(d["prev"], (1, 0, 2)))
        a_n, _ = cref.lisa_rows(d["q_lr"], d["k_lr"], d["v"], w1c, d["w2"], all_rows(3), prev_rows,
                                mix=cref.MIX_CONCAT, delta_scale=1.0)
        got = a_n[2, :, 0]
    else:
        a_n = npref.lisa_scores(d["q_lr"], d["k_lr"], w1c, d["w2"], d["prev"], mix=npref.MIX_CONCAT,
                                delta_scale=1.0)
        got = a_n[:, 2, 0]
    np.testing.assert_allclose(got, [3.0, 0.0], atol=1e-14)


# --------------------------------------------------------------------------------------
# 2. Softmax invariants: rows sum to one, nothing above the causal diagonal.
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("Lq,Lk", [(7, 7), (5, 9), (1, 6)])
def test_softmax_rows_sum_to_one_and_causal_zero(Lq, Lk):
    g = rng(1)
    H, Hkv, dk, r, F = 4, 2, 3, 2, 8
    q_lr, k_lr = g.normal(size=(H, Lq, r)), g.normal(size=(Hkv, Lk, r))
    v = g.normal(size=(Hkv, Lk, dk))
    w1, w2 = g.normal(size=(H, F)), g.normal(size=(F, H))
    prev = g.normal(size=(Lq, H, Lk))
    _, _, p = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(Lq), prev, want_probs=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-12)
    for i in range(Lq):
        nv = i + 1 + Lk - Lq
        assert np.all(p[i, :, nv:] == 0.0)
        assert np.all(p[i, :, :nv] > 0.0)
    _, _, p2 = npref.lisa_layer(q_lr, k_lr, v, w1, w2, np.transpose(prev, (1, 0, 2)))
    np.testing.assert_allclose(np.transpose(p2, (1, 0, 2)), p, atol=1e-13)


# --------------------------------------------------------------------------------------
# 3. Identity FFN + zero correction == textbook attention from library routines.
# --------------------------------------------------------------------------------------
def textbook_attention(q, k, v):
    """softmax(Q K^T / sqrt(d)) V with scipy's softmax and numpy's matmul, per head, causal
    by slicing (row i uses keys 0..i)."""
    H, L, dk = q.shape
    out = np.zeros((L, H, v.shape[-1]))
    for h in range(H):
        for i in range(L):
            s = (k[h, :i + 1] @ q[h, i]) / math.sqrt(dk)
            out[i, h] = scipy.special.softmax(s) @ v[h, :i + 1]
    return out


@pytest.mark.parametrize("impl", ["c", "numpy"])
def test_identity_ffn_zero_correction_is_standard_attention(impl):
    g = rng(2)
    H, L, dk, r = 3, 6, 4, 2
    F = 2 * H + 1
    q, k, v = g.normal(size=(H, L, dk)), g.normal(size=(H, L, dk)), g.normal(size=(H, L, dk))
    w1, w2 = identity_ffn(H, F)
    q_lr = np.zeros((H, L, r))
    k_lr = g.normal(size=(H, L, r))
    want = textbook_attention(q, k, v)
    if impl == "c":
        prev = cref.std_scores_rows(q, k, all_rows(L))
        a_n, out = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev)
        assert np.array_equal(a_n, prev)          # the sharing itself is exact
    else:
        prev = npref.std_scores(q, k)
        a_n, out, _ = npref.lisa_layer(q_lr, k_lr, v, w1, w2, prev)
        assert np.array_equal(a_n, prev)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-13)


def test_std_scores_match_library_matmul():
    g = rng(3)
    H, Hkv, Lq, Lk, dk = 4, 2, 5, 8, 6
    q, k = g.normal(size=(H, Lq, dk)), g.normal(size=(Hkv, Lk, dk))
    got = cref.std_scores_rows(q, k, all_rows(Lq))
    for h in range(H):
        full = (q[h] @ k[h // 2].T) / math.sqrt(dk)
        for i in range(Lq):
            nv = i + 1 + Lk - Lq
            np.testing.assert_allclose(got[i, h, :nv], full[i, :nv], atol=1e-14)
            assert np.all(got[i, h, nv:] == 0)


# --------------------------------------------------------------------------------------
# 4. The low-rank correction (Eq. 3).
# --------------------------------------------------------------------------------------
def test_a_delta_is_brute_force_triple_loop():
    g = rng(4)
    H, L, r, F = 2, 4, 3, 4
    q_lr, k_lr = g.normal(size=(H, L, r)), g.normal(size=(H, L, r))
    w1, w2 = np.zeros((H, F)), np.zeros((F, H))          # FFN contributes exactly zero
    prev = g.normal(size=(L, H, L))
    v = g.normal(size=(H, L, 2))
    a_n, _ = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev)
    for h in range(H):
        for i in range(L):
            for j in range(i + 1):
                s = 0.0
                for t in range(r):
                    s += q_lr[h][i][t] * k_lr[h][j][t]
                assert abs(a_n[i, h, j] - s / math.sqrt(r)) < 1e-14


def test_full_rank_correction_reduces_to_standard_scores():
    """With r = d_k and the same projections, Eq. 3 is Eq. 2's bracketed term."""
    g = rng(5)
    H, L, dk, F = 3, 5, 4, 6
    q, k = g.normal(size=(H, L, dk)), g.normal(size=(H, L, dk))
    std = cref.std_scores_rows(q, k, all_rows(L))
    a_n, _ = cref.lisa_rows(q, k, g.normal(size=(H, L, 2)), np.zeros((H, F)), np.zeros((F, H)),
                            all_rows(L), np.zeros((L, H, L)))
    np.testing.assert_allclose(a_n, std, atol=1e-14)


def test_add_mode_is_affine_in_the_correction():
    g = rng(6)
    H, Hkv, L, r, F, dk = 4, 2, 6, 3, 8, 2
    q_lr, k_lr = g.normal(size=(H, L, r)), g.normal(size=(Hkv, L, r))
    v = g.normal(size=(Hkv, L, dk))
    w1, w2 = g.normal(size=(H, F)), g.normal(size=(F, H))
    prev = g.normal(size=(L, H, L))
    a_full, _ = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev)
    a_ffn, _ = cref.lisa_rows(np.zeros_like(q_lr), k_lr, v, w1, w2, all_rows(L), prev)
    a_delta, _ = cref.lisa_rows(q_lr, k_lr, v, np.zeros_like(w1), w2, all_rows(L), prev)
    np.testing.assert_allclose(a_full - a_ffn, a_delta, atol=1e-13)
    # and the FFN part is the library expression relu(x W1) W2 on the head axis
    for i in range(L):
        for j in range(i + 1):
            x = prev[i, :, j]
            np.testing.assert_allclose(a_ffn[i, :, j], np.maximum(x @ w1, 0) @ w2, atol=1e-13)


def test_concat_mode_against_add_mode_on_stacked_heads():
    """FFN([A_prev; A_delta]) with W1 [2H,F] equals an ADD-mode layer over 2H 'heads' whose
    previous scores are the stacked tensor, with zero correction, restricted to H outputs."""
    g = rng(7)
    H, L, r, F, dk = 3, 5, 2, 7, 2
    q_lr, k_lr = g.normal(size=(H, L, r)), g.normal(size=(H, L, r))
    v = g.normal(size=(H, L, dk))
    w1, w2 = g.normal(size=(2 * H, F)), g.normal(size=(F, H))
    prev = g.normal(size=(L, H, L))
    a_cat, _ = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev, mix=cref.MIX_CONCAT)
    a_delta, _ = cref.lisa_rows(q_lr, k_lr, v, np.zeros((H, F)), np.zeros((F, H)), all_rows(L),
                                np.zeros_like(prev))
    stacked = np.concatenate([prev, a_delta], axis=1)               # [L, 2H, L]
    w2_wide = np.concatenate([w2, np.zeros((F, H))], axis=1)        # [F, 2H]
    zq = np.zeros((2 * H, L, r))
    a_ref, _ = cref.lisa_rows(zq, np.zeros((2 * H, L, r)), np.zeros((2 * H, L, dk)), w1, w2_wide,
                              all_rows(L), stacked)
    for i in range(L):
        np.testing.assert_allclose(a_cat[i, :, :i + 1], a_ref[i, :H, :i + 1], atol=1e-13)
    # zeroing W1's A_delta rows removes the correction entirely
    w1z = w1.copy()
    w1z[H:] = 0
    a_z, _ = cref.lisa_rows(q_lr, k_lr, v, w1z, w2, all_rows(L), prev, mix=cref.MIX_CONCAT)
    a_add0, _ = cref.lisa_rows(np.zeros_like(q_lr), k_lr, v, w1[:H], w2, all_rows(L), prev)
    np.testing.assert_allclose(a_z, a_add0, atol=1e-13)


# --------------------------------------------------------------------------------------
# 5. The worked head-permutation example of Sec. 5.1.
# --------------------------------------------------------------------------------------
def load_permutation():
    pairs = []
    with open(os.path.join(GOLDEN, "head_permutation_h3.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                s, t = line.split()
                pairs.append((int(s) - 1, int(t) - 1))
    return pairs


@pytest.mark.parametrize("impl", ["c", "numpy"])
def test_permutation_ffn_rearranges_heads(impl):
    pairs = load_permutation()
    assert sorted(p[0] for p in pairs) == [0, 1, 2]
    H, L, dk, r = 3, 5, 2, 2
    perm = np.zeros((H, H))
    for s, t in pairs:
        perm[s, t] = 1.0                      # x @ perm moves source head s to slot t
    F = 2 * H
    w1 = np.concatenate([perm, -perm], axis=1)
    w2 = np.concatenate([np.eye(H), -np.eye(H)], axis=0)
    g = rng(8)
    q, k = g.normal(size=(H, L, dk)), g.normal(size=(H, L, dk))
    v_shared = np.repeat(g.normal(size=(1, L, dk)), H, axis=0)   # same V for all heads
    q_lr, k_lr = np.zeros((H, L, r)), np.zeros((H, L, r))
    if impl == "c":
        prev = cref.std_scores_rows(q, k, all_rows(L))
        a_n, out, p = cref.lisa_rows(q_lr, k_lr, v_shared, w1, w2, all_rows(L), prev, want_probs=True)
        _, p_prev = cref.softmax_v_rows(v_shared, all_rows(L), prev, L, want_probs=True)
        out_prev = cref.softmax_v_rows(v_shared, all_rows(L), prev, L)
        for s, t in pairs:
            assert np.array_equal(a_n[:, t], prev[:, s])
            assert np.array_equal(p[:, t], p_prev[:, s])
            assert np.array_equal(out[:, t], out_prev[:, s])
    else:
        prev = npref.std_scores(q, k)
        a_n, out, p = npref.lisa_layer(q_lr, k_lr, v_shared, w1, w2, prev)
        out_prev, p_prev = npref.softmax_v(prev, v_shared)
        for s, t in pairs:
            assert np.array_equal(a_n[t], prev[s])
            assert np.array_equal(p[t], p_prev[s])
            assert np.array_equal(out[:, t], out_prev[:, s])


# --------------------------------------------------------------------------------------
# 6. Softmax * V closed forms.
# --------------------------------------------------------------------------------------
def test_uniform_scores_give_running_mean_of_values():
    g = rng(9)
    H, L, dk = 2, 7, 3
    v = g.normal(size=(H, L, dk))
    scores = np.full((L, H, L), 0.37)
    out = cref.softmax_v_rows(v, all_rows(L), scores, L)
    for i in range(L):
        np.testing.assert_allclose(out[i], v[:, :i + 1].mean(axis=1), atol=1e-14)


def test_dominant_score_selects_its_value_row():
    g = rng(10)
    H, L, dk = 2, 6, 3
    v = g.normal(size=(H, L, dk))
    scores = np.zeros((L, H, L))
    jstar = [0, 0, 1, 3, 2, 4]
    for i in range(L):
        scores[i, :, jstar[i]] = 800.0            # exp(-800) underflows to exactly 0
    out = cref.softmax_v_rows(v, all_rows(L), scores, L)
    for i in range(L):
        np.testing.assert_array_equal(out[i], v[:, jstar[i]])


def test_softmax_is_shift_invariant_and_handles_large_scores():
    g = rng(11)
    H, L, dk = 2, 5, 2
    v = g.normal(size=(H, L, dk))
    s = g.normal(size=(L, H, L))
    a = cref.softmax_v_rows(v, all_rows(L), s, L)
    b = cref.softmax_v_rows(v, all_rows(L), s + 5000.0, L)
    np.testing.assert_allclose(a, b, atol=1e-9)


# --------------------------------------------------------------------------------------
# 7. Structure: GQA, decode, row independence, C vs numpy.
# --------------------------------------------------------------------------------------
def test_gqa_equals_mha_with_repeated_kv():
    g = rng(12)
    H, Hkv, L, r, dk, F = 6, 2, 5, 2, 3, 12
    q_lr, k_lr = g.normal(size=(H, L, r)), g.normal(size=(Hkv, L, r))
    v = g.normal(size=(Hkv, L, dk))
    w1, w2 = g.normal(size=(H, F)), g.normal(size=(F, H))
    prev = g.normal(size=(L, H, L))
    a1, o1 = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev)
    rep = lambda x: np.concatenate([x[kv:kv + 1] for kv in range(Hkv) for _ in range(H // Hkv)], 0)
    a2, o2 = cref.lisa_rows(q_lr, rep(k_lr), rep(v), w1, w2, all_rows(L), prev)
    assert np.array_equal(a1, a2) and np.array_equal(o1, o2)
    q = g.normal(size=(H, L, 4))
    k = g.normal(size=(Hkv, L, 4))
    assert np.array_equal(cref.std_scores_rows(q, k, all_rows(L)),
                          cref.std_scores_rows(q, rep(k), all_rows(L)))


def test_decode_step_equals_last_prefill_row():
    g = rng(13)
    H, Hkv, L, r, dk, F = 4, 2, 9, 3, 4, 8
    q_lr, k_lr = g.normal(size=(H, L, r)), g.normal(size=(Hkv, L, r))
    v = g.normal(size=(Hkv, L, dk))
    w1, w2 = g.normal(size=(H, F)), g.normal(size=(F, H))
    prev = g.normal(size=(L, H, L))
    a_pre, o_pre = cref.lisa_rows(q_lr, k_lr, v, w1, w2, [L - 1], prev[L - 1:L])
    a_dec, o_dec = cref.lisa_rows(q_lr[:, L - 1:L], k_lr, v, w1, w2, [0], prev[L - 1:L])
    assert np.array_equal(a_pre, a_dec) and np.array_equal(o_pre, o_dec)


def test_rows_are_independent_of_the_request_set():
    g = rng(14)
    H, L, r, dk, F = 2, 8, 2, 2, 4
    q_lr, k_lr, v = g.normal(size=(H, L, r)), g.normal(size=(H, L, r)), g.normal(size=(H, L, dk))
    w1, w2 = g.normal(size=(H, F)), g.normal(size=(F, H))
    prev = g.normal(size=(L, H, L))
    a_all, o_all = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev)
    pick = [6, 1, 3]
    a_s, o_s = cref.lisa_rows(q_lr, k_lr, v, w1, w2, pick, prev[pick])
    assert np.array_equal(a_s, a_all[pick]) and np.array_equal(o_s, o_all[pick])


@pytest.mark.parametrize("mix", [0, 1])
@pytest.mark.parametrize("Lq,Lk,H,Hkv", [(12, 12, 8, 8), (5, 11, 8, 2), (1, 17, 6, 3)])
def test_c_and_numpy_oracles_agree(mix, Lq, Lk, H, Hkv):
    g = rng(100 + mix + Lq)
    r, dk, F = 5, 8, 2 * H + 3
    q_lr, k_lr = g.normal(size=(H, Lq, r)), g.normal(size=(Hkv, Lk, r))
    v = g.normal(size=(Hkv, Lk, dk))
    Din = 2 * H if mix else H
    w1, w2 = g.normal(size=(Din, F)) * 0.3, g.normal(size=(F, H)) * 0.3
    prev = g.normal(size=(H, Lq, Lk))
    a_c, o_c, p_c = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(Lq),
                                   np.ascontiguousarray(np.transpose(prev, (1, 0, 2))), mix=mix,
                                   want_probs=True)
    a_n, o_n, p_n = npref.lisa_layer(q_lr, k_lr, v, w1, w2, prev, mix=mix)
    np.testing.assert_allclose(np.transpose(a_c, (1, 0, 2)), a_n, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(np.transpose(p_c, (1, 0, 2)), p_n, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(o_c, o_n, rtol=1e-12, atol=1e-12)


def test_oracle_rejects_inconsistent_shapes():
    with pytest.raises((ValueError, AssertionError)):
        cref.std_scores_rows(np.zeros((3, 2, 2)), np.zeros((2, 2, 2)), [0])   # H % Hkv != 0


# --------------------------------------------------------------------------------------
# 8. Numbers printed in the paper that fix shapes (App. C.1, Sec. 5.1, Sec. 5.2).
# --------------------------------------------------------------------------------------
def load_kv(name):
    d = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, val = line.split()
                d[k] = int(val)
    return d


def test_printed_shapes_fix_per_head_rank_and_gqa_key_heads():
    s = load_kv("appendix_shapes.txt")
    r, dk = s["paper_r"], s["paper_dk"]
    assert s["llama3_8b_wq_cols"] == 32 * r            # r is per head
    assert s["llama3_8b_wk_cols"] == 8 * r             # K_LR has the KV heads of GQA
    assert s["llama2_7b_wk_cols"] == 32 * r
    assert s["llama2_13b_w_cols"] == 40 * r
    assert s["ffn1_rows"] == 2 * 32 and s["ffn2_cols"] == 32 and s["ffn1_cols"] == s["ffn2_rows"]
    per_layer = (s["llama3_8b_wq_rows"] * (s["llama3_8b_wq_cols"] + s["llama3_8b_wk_cols"])
                 + s["ffn1_rows"] * s["ffn1_cols"] + s["ffn2_rows"] * s["ffn2_cols"])
    total = s["llama3_8b_lisa_layers"] * per_layer
    assert round(total / 1e6) == s["llama3_8b_trained_params_millions"]
    assert round(dk / r) == 6                          # "compresses Q, K by 6x"


# --------------------------------------------------------------------------------------
# 9. Projection front end: Q_LR = X W^Q_LR, K_LR = X W^K_LR (factors of Eq. 3), V = X W^V
#    (Eq. 1), rotary position embedding of the LLaMA models of Sec. 5.3 on Q_LR / K_LR.
# --------------------------------------------------------------------------------------
def test_projection_without_rotation_is_a_library_matmul():
    g = rng(90)
    L, D, H, Hkv, r, dk = 7, 24, 4, 2, 6, 8
    x = g.standard_normal((L, D))
    w = g.standard_normal((H * r + Hkv * r + Hkv * dk, D))
    q, k, v = cref.project_rows(x, w, all_rows(L), H, Hkv, r, dk)
    y = x @ w.T
    np.testing.assert_allclose(q.reshape(L, -1), y[:, :H * r], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(k.reshape(L, -1), y[:, H * r:(H + Hkv) * r], rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(v.reshape(L, -1), y[:, (H + Hkv) * r:], rtol=1e-12, atol=1e-12)
    # feature f of head h is row h*r + f of the weight: a one-hot weight picks it out
    w1 = np.zeros_like(w)
    w1[2 * r + 3, 5] = 1.0
    q1, k1, v1 = cref.project_rows(x, w1, all_rows(L), H, Hkv, r, dk)
    assert np.count_nonzero(k1) == 0 and np.count_nonzero(v1) == 0
    np.testing.assert_array_equal(q1[:, 2, 3], x[:, 5])
    assert np.count_nonzero(q1) == np.count_nonzero(x[:, 5])


def test_rotary_embedding_unit_vectors_give_cos_and_sin():
    """r = 4, theta = 10^4: frequencies 1 and 10^-2; identity weights make Q_LR = X.
    e_0 -> (cos p, 0, sin p, 0); e_2 -> (-sin p, 0, cos p, 0); e_1 -> (0, cos p/100, 0, sin p/100):
    fixes the pairing (t, t + r/2), the sense of rotation and the exponent -2t/r."""
    r, dk, L = 4, 2, 6
    D = r
    w = np.zeros((r + r + dk, D))
    w[:r] = np.eye(r)
    w[r:2 * r] = np.eye(r)
    for e, expect in (
        (0, lambda p: [math.cos(p), 0.0, math.sin(p), 0.0]),
        (2, lambda p: [-math.sin(p), 0.0, math.cos(p), 0.0]),
        (1, lambda p: [0.0, math.cos(p / 100.0), 0.0, math.sin(p / 100.0)]),
        (3, lambda p: [0.0, -math.sin(p / 100.0), 0.0, math.cos(p / 100.0)]),
    ):
        x = np.zeros((L, D))
        x[:, e] = 1.0
        q, k, v = cref.project_rows(x, w, all_rows(L), 1, 1, r, dk, theta=1.0e4, pos0=3)
        want = np.array([expect(3 + i) for i in range(L)])
        np.testing.assert_allclose(q[:, 0, :], want, rtol=0, atol=1e-14)
        np.testing.assert_allclose(k[:, 0, :], want, rtol=0, atol=1e-14)
        assert np.count_nonzero(v) == 0                      # V is never rotated


def test_rotary_embedding_is_a_rotation_that_depends_on_relative_position():
    g = rng(91)
    L, D, H, Hkv, r, dk = 12, 10, 4, 2, 6, 4
    x = np.tile(g.standard_normal((1, D)), (L, 1))           # the same token at every position
    w = g.standard_normal((H * r + Hkv * r + Hkv * dk, D))
    q0, k0, v0 = cref.project_rows(x, w, all_rows(L), H, Hkv, r, dk)
    q, k, v = cref.project_rows(x, w, all_rows(L), H, Hkv, r, dk, theta=500000.0)
    np.testing.assert_array_equal(v, v0)
    np.testing.assert_allclose(q[0], q0[0], rtol=0, atol=1e-15)          # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(q, axis=-1), np.linalg.norm(q0, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(np.linalg.norm(k, axis=-1), np.linalg.norm(k0, axis=-1), rtol=1e-13)
    # <q_i, k_j> is a function of i - j
    s = np.einsum("ihr,jhr->hij", q[:, :Hkv], k)
    for d in range(-3, 4):
        diag = np.stack([np.diagonal(s[h], offset=d) for h in range(Hkv)])
        np.testing.assert_allclose(diag, np.repeat(diag[:, :1], diag.shape[1], axis=1),
                                   rtol=1e-11, atol=1e-12)
    assert np.abs(s[0, 0, 0] - s[0, 0, 5]) > 1e-3            # and does depend on it
    # a position offset shifts the rows
    q3, k3, _ = cref.project_rows(x, w, all_rows(L - 3), H, Hkv, r, dk, theta=500000.0, pos0=3)
    np.testing.assert_allclose(q3, q[3:], rtol=0, atol=1e-13)
    np.testing.assert_allclose(k3, k[3:], rtol=0, atol=1e-13)


def test_projection_rows_are_independent_of_the_request_set():
    g = rng(92)
    L, D, H, Hkv, r, dk = 9, 16, 2, 1, 4, 8
    x = g.standard_normal((L, D))
    w = g.standard_normal((H * r + Hkv * r + Hkv * dk, D))
    qa, ka, va = cref.project_rows(x, w, all_rows(L), H, Hkv, r, dk, theta=1.0e4, pos0=2)
    qs, ks, vs = cref.project_rows(x, w, [7, 1], H, Hkv, r, dk, theta=1.0e4, pos0=2)
    np.testing.assert_array_equal(qs, qa[[7, 1]])
    np.testing.assert_array_equal(ks, ka[[7, 1]])
    np.testing.assert_array_equal(vs, va[[7, 1]])
    with pytest.raises(ValueError):
        cref.project_rows(x[:, :15], np.zeros((3 + 3 + dk, 15)), [0], 1, 1, 3, dk, theta=1.0e4)


# --------------------------------------------------------------------------------------
# 10. Variants of the alignment module: SiLU and the single-layer FFN (Sec. 5.7), LiSA_plus
#     (Sec. 5.5: A_{n-1} + A_delta) and direct sharing (Sec. 4: A_n = A_{n-1}).
# --------------------------------------------------------------------------------------
def variant_problem(seed, H=4, Hkv=2, L=6, r=3, dk=5, F=7):
    g = rng(seed)
    q_lr = g.standard_normal((H, L, r))
    k_lr = g.standard_normal((Hkv, L, r))
    v = g.standard_normal((Hkv, L, dk))
    prev = g.standard_normal((L, H, L))                   # rows layout [n,H,Lk]
    return g, q_lr, k_lr, v, prev, H, Hkv, L, r, dk, F


def brute_a_delta(q_lr, k_lr, H, Hkv, L, r):
    ad = np.zeros((L, H, L))
    for i in range(L):
        for h in range(H):
            for j in range(L):
                ad[i, h, j] = sum(q_lr[h, i, t] * k_lr[h // (H // Hkv), j, t] for t in range(r)) / math.sqrt(r)
    return ad


def causal_mask(L):
    return np.tril(np.ones((L, L), dtype=bool))[:, None, :]     # [i,1,j]


@pytest.mark.parametrize("mix", [cref.MIX_ADD, cref.MIX_CONCAT])
def test_silu_ffn_matches_library_sigmoid(mix):
    g, q_lr, k_lr, v, prev, H, Hkv, L, r, dk, F = variant_problem(100)
    Din = 2 * H if mix == cref.MIX_CONCAT else H
    w1, w2 = g.standard_normal((Din, F)), g.standard_normal((F, H))
    a_n, _ = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev, mix=mix, act=cref.ACT_SILU)
    ad = brute_a_delta(q_lr, k_lr, H, Hkv, L, r)
    x = np.moveaxis(prev, 1, -1)                                  # [i,j,h]
    if mix == cref.MIX_CONCAT:
        x = np.concatenate([x, np.moveaxis(ad, 1, -1)], axis=-1)
    pre = x @ w1
    y = (pre * scipy.special.expit(pre)) @ w2
    want = np.moveaxis(y, -1, 1) + (ad if mix == cref.MIX_ADD else 0.0)
    np.testing.assert_allclose(a_n, np.where(causal_mask(L), want, 0.0), rtol=1e-12, atol=1e-12)
    # and it is not ReLU: a negative pre-activation leaks through
    a_relu, _ = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev, mix=mix, act=cref.ACT_RELU)
    assert np.abs(a_relu - a_n).max() > 1e-2


def test_silu_limits():
    """One head, F = 1, unit weights: y = silu(x); silu(0) = 0, silu(40) = 40, silu(-40) = 0 to 1e-15."""
    L = 3
    prev = np.zeros((L, 1, L))
    prev[0, 0, 0], prev[1, 0, 1], prev[2, 0, 2] = 0.0, 40.0, -40.0
    z = np.zeros((1, L, 2))
    a_n, _ = cref.lisa_rows(z, z, np.ones((1, L, 1)), np.ones((1, 1)), np.ones((1, 1)), all_rows(L), prev,
                            act=cref.ACT_SILU)
    assert a_n[0, 0, 0] == 0.0
    assert abs(a_n[1, 0, 1] - 40.0) < 1e-12
    assert abs(a_n[2, 0, 2]) < 1e-12


@pytest.mark.parametrize("mix", [cref.MIX_ADD, cref.MIX_CONCAT])
def test_single_layer_ffn_is_one_library_matmul(mix):
    g, q_lr, k_lr, v, prev, H, Hkv, L, r, dk, _ = variant_problem(101)
    Din = 2 * H if mix == cref.MIX_CONCAT else H
    w1 = g.standard_normal((Din, H))
    a_n, out = cref.lisa_rows(q_lr, k_lr, v, w1, None, all_rows(L), prev, mix=mix, act=cref.ACT_SINGLE)
    ad = brute_a_delta(q_lr, k_lr, H, Hkv, L, r)
    x = np.moveaxis(prev, 1, -1)
    if mix == cref.MIX_CONCAT:
        x = np.concatenate([x, np.moveaxis(ad, 1, -1)], axis=-1)
    want = np.moveaxis(x @ w1, -1, 1) + (ad if mix == cref.MIX_ADD else 0.0)
    np.testing.assert_allclose(a_n, np.where(causal_mask(L), want, 0.0), rtol=1e-12, atol=1e-12)
    # a two-layer FFN with an identity second layer and no activation clipping is the same map:
    # with the [I,-I] / [I;-I] trick the ReLU network reproduces it exactly
    w1r = np.concatenate([w1, -w1], axis=1)
    w2r = np.concatenate([np.eye(H), -np.eye(H)], axis=0)
    a_two, out_two = cref.lisa_rows(q_lr, k_lr, v, w1r, w2r, all_rows(L), prev, mix=mix)
    np.testing.assert_allclose(a_n, a_two, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out, out_two, rtol=1e-12, atol=1e-12)
    with pytest.raises(ValueError):                                # W1 must be [Din, H]
        cref.lisa_rows(q_lr, k_lr, v, g.standard_normal((Din, H + 1)), None, all_rows(L), prev, mix=mix,
                       act=cref.ACT_SINGLE)


def test_plus_variant_adds_the_brute_force_correction():
    g, q_lr, k_lr, v, prev, H, Hkv, L, r, dk, _ = variant_problem(102)
    a_n, out = cref.lisa_rows(q_lr, k_lr, v, None, None, all_rows(L), prev, mix=cref.MIX_PLUS)
    want = prev + brute_a_delta(q_lr, k_lr, H, Hkv, L, r)
    np.testing.assert_allclose(a_n, np.where(causal_mask(L), want, 0.0), rtol=1e-12, atol=1e-12)
    # equals the ADD layer whose FFN is the identity
    w1, w2 = identity_ffn(H, 2 * H)
    a_add, out_add = cref.lisa_rows(q_lr, k_lr, v, w1, w2, all_rows(L), prev)
    np.testing.assert_allclose(a_n, a_add, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out, out_add, rtol=1e-12, atol=1e-12)


def test_direct_sharing_is_textbook_attention_on_the_previous_scores():
    g, q_lr, k_lr, v, prev, H, Hkv, L, r, dk, _ = variant_problem(103)
    a_n, out = cref.lisa_rows(None, None, v, None, None, all_rows(L), prev, mix=cref.MIX_SHARE, Lq=L)
    np.testing.assert_array_equal(a_n, np.where(causal_mask(L), prev, 0.0))
    masked = np.where(causal_mask(L), prev, -np.inf)
    p = scipy.special.softmax(masked, axis=-1)                     # [i,h,j]
    vv = np.repeat(v, H // Hkv, axis=0)                            # [h,j,d]
    want = np.einsum("ihj,hjd->ihd", p, vv)
    np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-12)
    # passing Q_LR / K_LR changes nothing
    a2, out2 = cref.lisa_rows(q_lr, k_lr, v, None, None, all_rows(L), prev, mix=cref.MIX_SHARE)
    np.testing.assert_array_equal(a2, a_n)
    np.testing.assert_array_equal(out2, out)


# ---------------------------------------------------------------------------------------
# knowledge-distillation regression term (Sec. 5.1 "Training strategy", App. C.1 Huber loss)
# ---------------------------------------------------------------------------------------
def test_huber_loss_values_worked_by_hand():
    """delta = 1: differences 0.5, -0.5, 1, 2, -3 give 1/8, 1/8, 1/2 (both branches agree at
    |d| = delta), 3/2, 5/2; delta = 2: a difference of 3 gives 2 (3 - 1) = 4."""
    from oracle import npref
    a = np.array([0.5, 1.0, 3.0, 5.0, -1.0])
    b = np.array([0.0, 1.5, 2.0, 3.0, 2.0])
    assert np.allclose(npref.huber(a, b, 1.0), [0.125, 0.125, 0.5, 1.5, 2.5], rtol=0, atol=1e-15)
    assert npref.huber(3.0, 0.0, 2.0) == 4.0
    assert npref.huber(1.25, 1.25, 1.0) == 0.0


def test_huber_loss_matches_the_library_routine_and_its_two_regimes():
    from scipy.special import huber as sp_huber
    from oracle import npref
    rng = np.random.default_rng(5)
    a, b = rng.normal(size=4000) * 2, rng.normal(size=4000) * 2
    for delta in (0.5, 1.0, 3.0):
        assert np.allclose(npref.huber(a, b, delta), sp_huber(delta, a - b), rtol=1e-14, atol=0)
    small = np.abs(a - b) <= 1.0                            # quadratic regime = half the squared error
    assert np.allclose(npref.huber(a, b)[small], 0.5 * (a - b)[small] ** 2)
    assert np.allclose(npref.huber(a, b)[~small], np.abs(a - b)[~small] - 0.5)   # linear regime, delta = 1
    assert np.array_equal(npref.huber(a, b), npref.huber(b, a))                  # symmetric
    # L_delta(d) = delta^2 L_1(d / delta)
    assert np.allclose(npref.huber(a, b, 3.0), 9.0 * npref.huber(a / 3.0, b / 3.0, 1.0))


def test_kd_loss_is_the_mean_over_visible_entries_only():
    from oracle import npref
    rng = np.random.default_rng(6)
    H, Lq, Lk = 3, 5, 7
    s, t = rng.normal(size=(2, H, Lq, Lk)), rng.normal(size=(2, H, Lq, Lk))
    vis = npref.visible(Lq, Lk)
    want = np.mean([npref.huber(s[b, h, i, j], t[b, h, i, j]) for b in range(2) for h in range(H)
                    for i in range(Lq) for j in range(Lk) if j <= i + Lk - Lq])
    assert abs(npref.kd_loss(s, t) - want) < 1e-15
    s2 = s.copy()
    s2[..., ~vis] = 1e9                                     # what a row cannot see does not count
    assert npref.kd_loss(s2, t) == npref.kd_loss(s, t)
    assert npref.kd_loss(s, s) == 0.0
    full = npref.kd_loss(s, t, causal=False)
    assert abs(full - npref.huber(s, t).mean()) < 1e-15
    # differences all below delta: half the mean squared error; all above: mean absolute error - 1/2
    assert abs(npref.kd_loss(t + 0.25, t) - 0.03125) < 1e-15
    assert abs(npref.kd_loss(t + 4.0, t) - 3.5) < 1e-12
