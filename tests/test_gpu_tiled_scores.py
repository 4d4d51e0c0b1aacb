"""The tiled score layout ([B,Lq/16,Lk/32,H,16,32], 1 KB per head and tile): the standard layer writes it, the
LiSA layer reads and writes it.  The row-major path is checked against the oracle elsewhere; here
the tiled path must give the same bits (same arithmetic, other addresses) on shapes that cover every
instantiation and launch geometry of the fused kernel, and is checked against the oracle directly
at the benchmark sizes."""
import numpy as np
import pytest
import torch

from paper_2408_01890_amd import lisa, synth
from tests import helpers as hp
from tests.test_gpu_parity import (DEV, FUSED_SHAPES, SLICE_SHAPES, STD_MFMA_SHAPES, check_prefill, log,
                                   tuned)  # noqa: F401  (tuned is a fixture)

pytestmark = pytest.mark.gpu


def visible_mask(Lq, Lk, causal, dev):
    m = torch.ones(Lq, Lk, dtype=torch.bool, device=dev)
    return m.tril(Lk - Lq) if causal else m


@pytest.mark.parametrize("case", STD_MFMA_SHAPES, ids=[c[0] for c in STD_MFMA_SHAPES])
def test_std_scores_tiled_equal_row_major(case):
    name, B, H, Hkv, Lq, Lk, causal = case
    dt = torch.bfloat16
    g = torch.Generator(device=DEV).manual_seed(29)
    q = torch.randn((B, H, Lq, 128), generator=g, device=DEV).to(dt)
    k = torch.randn((B, Hkv, Lk, 128), generator=g, device=DEV).to(dt)
    v = torch.randn((B, Hkv, Lk, 128), generator=g, device=DEV).to(dt)
    s_rm, o_rm = lisa.std_attn_scores(q, k, v, causal=causal)
    s_t, o_t = lisa.std_attn_scores(q, k, v, causal=causal, tiled=True)
    assert lisa.last_path() == "mfma_std"
    s_t2, _ = lisa.std_attn_scores(q, k, causal=causal, tiled=True)           # scores only
    torch.cuda.synchronize()
    assert s_t.shape == lisa.scores_shape(B, H, Lq, Lk, True)
    vis = visible_mask(Lq, Lk, causal, DEV)
    assert torch.equal(o_rm, o_t)
    assert torch.equal(lisa.untile_scores(s_t, Lq, Lk)[..., vis], s_rm[..., vis])
    assert torch.equal(lisa.untile_scores(s_t2, Lq, Lk)[..., vis], s_rm[..., vis])
    # tile_scores is the inverse on what is defined
    bits = s_rm.view(torch.int16)                      # (what lies above the diagonal is uninitialised)
    assert torch.equal(lisa.untile_scores(lisa.tile_scores(bits), Lq, Lk), bits)


def make_case(name, B, H, Hkv, Lq, Lk, r, F, seed, ffn="fan_in"):
    cfg = synth.LayerShape(name, "bf16", B, H, Hkv, Lk, 256, 128, r, F)
    inp = synth.make_prefill_inputs(cfg, seed, DEV, ffn=ffn)
    shift = Lk - Lq
    inp["q_lr"] = inp["q_lr"][:, :, shift:].contiguous()
    inp["q"] = inp["q"][:, :, shift:].contiguous()
    return cfg, inp


def both_layouts(inp, Lq, Lk, causal=True, **kw):
    """Two chained LiSA layers in both layouts; returns what must agree."""
    B, H = inp["q_lr"].shape[:2]
    prev_rm, _ = lisa.std_attn_scores(inp["q"], inp["k"], causal=causal)
    prev_t, _ = lisa.std_attn_scores(inp["q"], inp["k"], causal=causal, tiled=True)
    args = (inp["q_lr"], inp["k_lr"], inp["v"])
    o_rm, a_rm = lisa.lisa_attn_prefill(*args, prev_rm, inp["w1"], inp["w2"], causal=causal, **kw)
    path = lisa.last_path()
    o_t, a_t = lisa.lisa_attn_prefill(*args, prev_t, inp["w1"], inp["w2"], causal=causal, tiled=True, **kw)
    assert lisa.last_path() == path
    # second layer on the emitted A_n: what a stored tile holds above the diagonal must not matter
    o2_rm, _ = lisa.lisa_attn_prefill(*args, a_rm, inp["w1"], inp["w2"], causal=causal, write_scores=False, **kw)
    o2_t, _ = lisa.lisa_attn_prefill(*args, a_t, inp["w1"], inp["w2"], causal=causal, tiled=True,
                                     write_scores=False, **kw)
    torch.cuda.synchronize()
    vis = visible_mask(Lq, Lk, causal, DEV)
    assert bool(torch.isfinite(o_t).all()) and bool(torch.isfinite(o2_t).all())
    assert torch.equal(o_rm, o_t), "O differs between the layouts"
    assert torch.equal(lisa.untile_scores(a_t, Lq, Lk)[..., vis], a_rm[..., vis]), "A_n differs"
    assert torch.equal(o2_rm, o2_t), "second layer differs"
    return path, prev_t, o_t, a_t


TILED_CASES = (
    [(c[0], c[1], c[2], c[3], c[4], c[4], c[6], c[7], {}) for c in FUSED_SHAPES] +
    [(c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], {}) for c in SLICE_SHAPES] +
    [("h32_gqa_l520_pair", 1, 32, 8, 520, 520, 22, 64, dict(prefill_pair=1, prefill_split=1)),
     ("h32_gqa_l520_split4", 1, 32, 8, 520, 520, 22, 64, dict(prefill_pair=0, prefill_split=4)),
     ("h32_l520_groups4", 1, 32, 32, 520, 520, 22, 64, dict(prefill_groups=4)),
     ("h32_l520_groups1", 1, 32, 8, 520, 520, 22, 64, dict(prefill_groups=1)),
     ("h32_l520_groups2_pair", 1, 32, 32, 504, 520, 22, 64, dict(prefill_groups=2, prefill_pair=1)),
     ("h40_l328_slices2", 1, 40, 40, 328, 328, 22, 80, dict(prefill_slices=2, prefill_pair=1)),
     ("h8_l264_slices4", 2, 8, 8, 240, 264, 11, 64, dict(prefill_slices=4)),
     ("h16_l296_groups2", 1, 16, 4, 296, 296, 22, 64, dict(prefill_groups=2, prefill_split=2))])


@pytest.mark.parametrize("case", TILED_CASES, ids=[c[0] for c in TILED_CASES])
@pytest.mark.parametrize("causal", [True, False])
def test_lisa_prefill_tiled_equals_row_major(case, causal, tuned):
    name, B, H, Hkv, Lq, Lk, r, F, knobs = case
    if knobs:
        tuned(**knobs)
    log(f"[case] tiled scores {name} causal={causal} {knobs}")
    cfg, inp = make_case(name, B, H, Hkv, Lq, Lk, r, F, 41)
    path, *_ = both_layouts(inp, Lq, Lk, causal)
    assert path == "mfma_fused"


@pytest.mark.parametrize("variant", ["silu", "single", "plus", "share"])
def test_variants_on_the_fused_kernel_tiled(variant):
    cfg, inp = make_case("h32_l264_" + variant, 1, 32, 32, 264, 264, 22, 64, 43)
    H = 32
    g = torch.Generator(device=DEV).manual_seed(5)
    kw = {}
    if variant == "silu":
        kw = dict(act=lisa.ACT_SILU)
    elif variant == "single":
        inp["w1"] = (torch.randn((H, H), generator=g, device=DEV) / H ** 0.5).to(torch.bfloat16)
        inp["w2"] = None
        kw = dict(act=lisa.ACT_SINGLE)
    elif variant == "plus":
        inp["w1"] = inp["w2"] = None
        kw = dict(mix=lisa.MIX_PLUS)
    else:
        inp["w1"] = inp["w2"] = None
        kw = dict(mix=lisa.MIX_SHARE)
    path, *_ = both_layouts(inp, 264, 264, True, **kw)
    assert path == "mfma_fused"


CONCAT_TILED = [
    # name, B, H, Hkv, Lq, Lk, r, F, act
    ("paper_widths_l328", 1, 32, 32, 328, 328, 20, 256, "relu"),
    ("paper_widths_gqa_shift", 2, 32, 8, 200, 264, 20, 256, "relu"),
    ("h16_f128_l520", 1, 16, 16, 520, 520, 22, 128, "relu"),
    ("h24_f96_l136", 1, 24, 8, 136, 136, 16, 96, "relu"),
    ("h8_f64_silu_l264", 2, 8, 2, 264, 264, 11, 64, "silu"),
    ("h32_single_layer_l264", 1, 32, 32, 264, 264, 32, 0, "single"),
]


@pytest.mark.parametrize("case", CONCAT_TILED, ids=[c[0] for c in CONCAT_TILED])
@pytest.mark.parametrize("causal", [True, False])
def test_concat_pipeline_tiled_equals_row_major(case, causal):
    """CONCAT form (Sec. 5.1 overview, Sec. 5.3 widths) on the matrix cores: the scores kernel reads and
    writes tiles, the softmax / P V kernel reads them."""
    name, B, H, Hkv, Lq, Lk, r, F, act = case
    log(f"[case] tiled concat {name} causal={causal}")
    cfg = synth.LayerShape(name, "bf16", B, H, Hkv, Lk, 256, 128, r, max(F, 32))
    inp = synth.make_prefill_inputs(cfg, 53, DEV, mix="concat", ffn="fan_in")
    shift = Lk - Lq
    inp["q_lr"] = inp["q_lr"][:, :, shift:].contiguous()
    inp["q"] = inp["q"][:, :, shift:].contiguous()
    kw = dict(mix=lisa.MIX_CONCAT)
    if act == "silu":
        kw["act"] = lisa.ACT_SILU
    elif act == "single":                                   # LiSA_SL: one layer over the concatenation
        g = torch.Generator(device=DEV).manual_seed(7)
        inp["w1"] = (torch.randn((2 * H, H), generator=g, device=DEV) / (2 * H) ** 0.5).to(torch.bfloat16)
        inp["w2"] = None
        kw["act"] = lisa.ACT_SINGLE
    path, *_ = both_layouts(inp, Lq, Lk, causal, **kw)
    assert path == "mfma_scores"


def test_tiled_requests_outside_the_matrix_core_kernels_are_refused():
    cfg, inp = make_case("h32_l136", 1, 32, 32, 136, 136, 20, 160, 47)      # ADD with F = 160: not a fused shape
    prev_t, _ = lisa.std_attn_scores(inp["q"], inp["k"], tiled=True)
    with pytest.raises(lisa.LisaError) as e:
        lisa.lisa_attn_prefill(inp["q_lr"], inp["k_lr"], inp["v"], prev_t, inp["w1"], inp["w2"], tiled=True)
    assert e.value.status == -3
    cfg = synth.LayerShape("h40_concat", "bf16", 1, 40, 40, 136, 256, 128, 20, 256)   # CONCAT beyond 32 heads
    inp = synth.make_prefill_inputs(cfg, 47, DEV, mix="concat")
    prev_t, _ = lisa.std_attn_scores(inp["q"], inp["k"], tiled=True)
    with pytest.raises(lisa.LisaError) as e:
        lisa.lisa_attn_prefill(inp["q_lr"], inp["k_lr"], inp["v"], prev_t, inp["w1"], inp["w2"], tiled=True,
                               mix=lisa.MIX_CONCAT)
    assert e.value.status == -3
    q32 = torch.randn((1, 2, 40, 16), device=DEV)
    with pytest.raises(lisa.LisaError) as e:
        lisa.std_attn_scores(q32, q32, tiled=True)                          # fp32: generic kernels
    assert e.value.status == -3


def test_lisa_prefill_tiled_c2_full_size_all_rows_against_the_oracle():
    cfg = synth.C2
    inp = synth.make_prefill_inputs(cfg, synth.BASE_SEED + 2, DEV)
    prev, _ = lisa.std_attn_scores(inp["q"], inp["k"], tiled=True)
    out, scores = lisa.lisa_attn_prefill(inp["q_lr"], inp["k_lr"], inp["v"], prev, inp["w1"], inp["w2"],
                                         tiled=True)
    torch.cuda.synchronize()
    assert lisa.last_path() == "mfma_fused"
    rows = np.arange(cfg.L)
    ref_prev = hp.oracle_std_rows(inp["q"], inp["k"], 0, rows)
    assert hp.scores_row_rel_err(hp.gather_score_rows(prev, 0, rows, cfg.L), ref_prev, rows, cfg.L,
                                 cfg.L) <= hp.TOL[cfg.torch_dtype]
    check_prefill(cfg, inp, prev, out, scores, {0: rows}, tag="/tiled")


@pytest.mark.parametrize("cfg,ffn", [(synth.C3, "paper"), (synth.C3, "identity_noise"), (synth.C4, "paper")],
                         ids=["c3", "c3_identity_noise", "c4"])
def test_lisa_prefill_tiled_full_size_sampled_rows(cfg, ffn):
    """The launch configuration the bench times: tiled scores from the standard layer through the
    LiSA layer, sampled query rows against the oracle."""
    idx = 3 if cfg is synth.C3 else 4
    inp = synth.make_prefill_inputs(cfg, synth.BASE_SEED + idx, DEV, ffn=ffn)
    prev, _ = lisa.std_attn_scores(inp["q"], inp["k"], tiled=True)
    del inp["q"], inp["k"]
    out, scores = lisa.lisa_attn_prefill(inp["q_lr"], inp["k_lr"], inp["v"], prev, inp["w1"], inp["w2"],
                                         tiled=True)
    torch.cuda.synchronize()
    assert lisa.last_path() == "mfma_fused"
    per_b = 256 // cfg.B + 24
    rows_by_b = {b: synth.sample_rows(cfg.L, per_b, 100 + b) for b in range(cfg.B)}
    check_prefill(cfg, inp, prev, out, scores, rows_by_b, tag=f"/{ffn}/tiled")


@pytest.mark.parametrize("cfg", [synth.C3, synth.C4], ids=["c3", "c4"])
def test_std_layer_tiled_full_size_sampled_rows(cfg):
    """The standard layer (Eq. 1-2) as bench.py times it on the two large shapes: tiled scores and
    its own O, sampled query rows of every sequence against the oracle."""
    from oracle import cref
    idx = 3 if cfg is synth.C3 else 4
    inp = synth.make_prefill_inputs(cfg, synth.BASE_SEED + 30 + idx, DEV)
    scores, out = lisa.std_attn_scores(inp["q"], inp["k"], inp["v"], tiled=True)
    torch.cuda.synchronize()
    assert lisa.last_path() == "mfma_std"
    tol = hp.TOL[cfg.torch_dtype]
    ea = eo = 0.0
    for b in range(cfg.B):
        rows = synth.sample_rows(cfg.L, 64 // cfg.B + 8, 200 + b)
        ref = hp.oracle_std_rows(inp["q"], inp["k"], b, rows)
        ea = max(ea, hp.scores_row_rel_err(hp.gather_score_rows(scores, b, rows, cfg.L), ref, rows, cfg.L, cfg.L))
        o_ref = cref.softmax_v_rows(hp.f64(inp["v"][b]), rows, ref, cfg.L)
        eo = max(eo, hp.row_rel_err(hp.gather_out_rows(out, b, rows), o_ref))
    log(f"[parity] std mfma tiled {cfg.name}: err_scores={ea:.3e} err_out={eo:.3e} tol={tol:g}")
    assert max(ea, eo) <= tol


@pytest.mark.parametrize("ffn", ["paper", "fan_in"])
def test_concat_tiled_full_size_sampled_rows_against_the_oracle(ffn):
    """The paper's module at its own widths (Sec. 5.3: 64 -> 256 -> 32, r = 20) on the LLaMA2-7B shape,
    on tiled score tensors as bench.py times it."""
    cfg = synth.LayerShape("c2_concat_64_256_32_r20_tiled", "bf16", 1, 32, 32, 2048, 4096, 128, 20, 256)
    log(f"[case] prefill {cfg.name} ffn={ffn} sampled")
    inp = synth.make_prefill_inputs(cfg, synth.BASE_SEED + 21, DEV, mix="concat", ffn=ffn)
    prev, _ = lisa.std_attn_scores(inp["q"], inp["k"], tiled=True)
    out, scores = lisa.lisa_attn_prefill(inp["q_lr"], inp["k_lr"], inp["v"], prev, inp["w1"], inp["w2"],
                                         mix=lisa.MIX_CONCAT, tiled=True)
    torch.cuda.synchronize()
    assert lisa.last_path() == "mfma_scores"
    rows = synth.sample_rows(cfg.L, 280, 121)
    check_prefill(cfg, inp, prev, out, scores, {0: rows}, mix=1, tag=f"/{ffn}/tiled")
