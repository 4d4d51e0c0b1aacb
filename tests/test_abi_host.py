"""Host-only checks of the C ABI (no GPU, no compute call): the shared library loads, exports
every function include/lisa.h declares, rejects bad arguments before touching HIP, and its
size helpers equal the closed forms of the paper's memory analysis (Sec. 5.2)."""
import ctypes as C
import os
import re

import pytest

from paper_2408_01890_amd import lisa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = C.c_void_p(0x10000)          # non-NULL, 16-byte aligned, never dereferenced on the host
ODD = C.c_void_p(0x10008)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lisa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:int|size_t|const char\*)\s+(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = lisa.library()
    names = declared_functions()
    assert {"lisa_attn_prefill", "lisa_attn_decode", "std_attn_scores"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/lisa.h but not exported"
    assert set(names) == set(lisa.EXPORTS)


def test_desc_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "lisa.h")).read()
    body = re.search(r"typedef struct lisa_desc \{(.*?)\} lisa_desc;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(?:int32_t|float)\s+(\w+);", body)
    assert fields == [f[0] for f in lisa.Desc._fields_]
    assert C.sizeof(lisa.Desc) == 4 * len(fields)


def good_desc(**kw):
    base = dict(dtype=lisa.BF16, B=2, H=8, Hkv=4, Lq=16, Lk=16, d_k=64, r=11, F=32)
    base.update(kw)
    return lisa.make_desc(**base)


def call_prefill(desc, **over):
    args = dict(q_lr=FAKE, k_lr=FAKE, v=FAKE, prev=FAKE, w1=FAKE, w2=FAKE, out=FAKE, sout=FAKE,
                ws=FAKE, wsb=1 << 40)
    args.update(over)
    return lisa.library().lisa_attn_prefill(
        C.byref(desc), args["q_lr"], args["k_lr"], args["v"], args["prev"], args["w1"], args["w2"],
        args["out"], args["sout"], args["ws"], args["wsb"], None)


def test_prefill_rejects_bad_arguments_before_any_hip_call():
    assert lisa.supported(good_desc()) == 0
    assert call_prefill(good_desc(), q_lr=None) == -1                       # NULL
    assert call_prefill(good_desc(write_scores=1), sout=None) == -1
    assert call_prefill(good_desc(H=6)) == -2                               # H % Hkv
    assert call_prefill(good_desc(Lq=32, Lk=16)) == -2                      # causal needs Lk >= Lq
    assert call_prefill(good_desc(r=0)) == -2
    assert call_prefill(good_desc(dtype=1, d_k=512)) == -3                  # beyond kernel range
    assert call_prefill(good_desc(mix=7)) == -3
    assert call_prefill(good_desc(act=3)) == -3
    assert call_prefill(good_desc(), v=ODD) == -4                           # alignment
    assert call_prefill(good_desc(write_scores=0), ws=None, sout=None) == -5   # workspace
    assert call_prefill(good_desc(write_scores=0), wsb=16, sout=None) == -5
    d = good_desc(write_scores=1)
    assert call_prefill(d, prev=FAKE, sout=FAKE) == -2                      # aliasing
    assert lisa.library().lisa_attn_prefill(None, *([FAKE] * 9), 0, None) == -1


def test_decode_and_std_reject_bad_arguments():
    lib = lisa.library()
    d = good_desc(Lq=1, Lk=9, Lmax=8, write_scores=1)
    a = [FAKE] * 11
    assert lib.lisa_attn_decode(C.byref(d), *a, 0, None) == -2              # Lmax < Lk
    d = good_desc(Lq=2, Lk=9, Lmax=16, write_scores=1)
    assert lib.lisa_attn_decode(C.byref(d), *a, 0, None) == -2              # Lq must be 1
    d = good_desc(Lq=1, Lk=9, Lmax=16, write_scores=1)
    b = list(a)
    b[1] = None                                                             # k_lr_new without v_new
    assert lib.lisa_attn_decode(C.byref(d), *b, 0, None) == -1
    d = good_desc()
    assert lib.std_attn_scores(C.byref(d), FAKE, FAKE, None, None, None, None, 0, None) == -1
    assert lib.std_attn_scores(C.byref(d), FAKE, FAKE, FAKE, FAKE, None, None, 0, None) == -1
    assert lib.std_attn_scores(C.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None) == -5
    # decode form: a cache capacity below the attended length, or a capacity on a prefill call
    d = good_desc(Lq=1, Lk=9, Lmax=8)
    assert lib.std_attn_scores(C.byref(d), FAKE, FAKE, None, FAKE, None, None, 0, None) == -2
    d = good_desc(Lq=4, Lk=9, Lmax=16)
    assert lib.std_attn_scores(C.byref(d), FAKE, FAKE, None, FAKE, None, None, 0, None) == -2


def test_static_scratch_decode_rejects_what_does_not_fit_before_any_launch():
    B, H, Lk = 64, 32, 4097
    d = lisa.make_desc(lisa.BF16, B, H, H, 1, Lk, 128, 22, 64, write_scores=1, kcache_dim_major=1, Lmax=Lk)
    assert lisa.workspace_bytes(d, lisa.WS_DECODE) > (16 << 20)
    lib = lisa.library()
    ptrs = [C.c_void_p(0x10000 + 0x100 * i) for i in range(10)]             # distinct: no aliasing
    assert lib.lisa_attn_decode_static(C.byref(d), *ptrs, None) == -7
    assert "static" in lib.lisa_strerror(-7).decode()
    fits = lisa.make_desc(lisa.BF16, 30, H, H, 1, Lk, 128, 22, 64, write_scores=1, kcache_dim_major=1, Lmax=Lk)
    assert lisa.workspace_bytes(fits, lisa.WS_DECODE) <= (16 << 20)
    a = list(ptrs)
    a[5] = None                                                             # score_row_prev
    assert lib.lisa_attn_decode_static(C.byref(fits), *a, None) == -1       # other checks come first
    a = list(ptrs)
    a[4] = ODD
    assert lib.lisa_attn_decode_static(C.byref(fits), *a, None) == -4


def test_tune_set_accepts_known_knobs_only():
    lib = lisa.library()
    assert lib.lisa_tune_set(lisa.TUNE_PREFILL_SPLIT, 2) == 0
    d = good_desc(dtype=lisa.BF16, B=1, H=32, Hkv=32, Lq=2048, Lk=2048, d_k=128, r=22, F=64)
    two = lisa.workspace_bytes(d, lisa.WS_PREFILL)
    assert lib.lisa_tune_set(lisa.TUNE_PREFILL_SPLIT, 3) == 0               # not 1, 2 or 4: ignored
    auto = lisa.workspace_bytes(d, lisa.WS_PREFILL)
    assert lib.lisa_tune_set(lisa.TUNE_PREFILL_SPLIT, -1) == 0
    assert lisa.workspace_bytes(d, lisa.WS_PREFILL) == auto and two > 0
    assert lib.lisa_tune_set(99, 1) == -2 and lib.lisa_tune_set(-1, 1) == -2


def test_cache_fill_rejects_bad_arguments():
    lib = lisa.library()
    d = lisa.make_desc(lisa.BF16, 2, 8, 2, 1, 100, 128, 22, 0, kcache_dim_major=1, Lmax=128)
    assert lib.lisa_cache_fill(None, FAKE, FAKE, FAKE, FAKE, None) == -1
    assert lib.lisa_cache_fill(C.byref(d), FAKE, None, FAKE, FAKE, None) == -1
    short = lisa.make_desc(lisa.BF16, 2, 8, 2, 1, 100, 128, 22, 0, kcache_dim_major=1, Lmax=64)
    assert lib.lisa_cache_fill(C.byref(short), FAKE, FAKE, FAKE, FAKE, None) == -2
    layout = lisa.make_desc(lisa.BF16, 2, 8, 2, 1, 100, 128, 22, 0, kcache_dim_major=3, Lmax=128)
    assert lib.lisa_cache_fill(C.byref(layout), FAKE, FAKE, FAKE, FAKE, None) == -2
    wide = lisa.make_desc(lisa.BF16, 2, 8, 2, 1, 100, 256, 200, 0, kcache_dim_major=1, Lmax=128)
    assert lib.lisa_cache_fill(C.byref(wide), FAKE, FAKE, FAKE, FAKE, None) == -3
    assert lib.lisa_cache_fill(C.byref(d), FAKE, ODD, FAKE, FAKE, None) == -4
    assert lib.lisa_cache_fill(C.byref(d), FAKE, FAKE, ODD, FAKE, None) == -4
    many = lisa.make_desc(lisa.BF16, 70000, 8, 2, 1, 100, 128, 22, 0, kcache_dim_major=1, Lmax=128)
    assert lib.lisa_cache_fill(C.byref(many), FAKE, FAKE, FAKE, FAKE, None) == -3


def test_proj_desc_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "lisa.h")).read()
    body = re.search(r"typedef struct lisa_proj_desc \{(.*?)\} lisa_proj_desc;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(?:int32_t|float)\s+(\w+);", body)
    assert fields == [f[0] for f in lisa.ProjDesc._fields_]
    assert C.sizeof(lisa.ProjDesc) == 4 * len(fields)


def test_project_qkv_rejects_bad_arguments():
    lib = lisa.library()

    def desc(**kw):
        base = dict(dtype=lisa.BF16, B=2, L=16, d_model=256, H=8, Hkv=2, r=22, d_k=128, Lmax=32,
                    pos0=4, kcache_dim_major=0, rope_theta=10000.0)
        base.update(kw)
        return lisa.ProjDesc(*[base[f[0]] for f in lisa.ProjDesc._fields_])

    def call(d, *ptrs):
        ptrs = list(ptrs) + [FAKE] * (5 - len(ptrs))
        return lib.lisa_project_qkv(C.byref(d) if d is not None else None, *ptrs, None)

    assert call(None) == -1
    assert call(desc(), FAKE, None) == -1
    assert call(desc(L=0)) == -2
    assert call(desc(H=8, Hkv=3)) == -2
    assert call(desc(Lmax=19)) == -2                   # pos0 + L = 20 does not fit
    assert call(desc(pos0=-1)) == -2
    assert call(desc(r=21)) == -2                      # rotary pairs need an even r
    assert call(desc(rope_theta=-1.0)) == -2
    assert call(desc(kcache_dim_major=2)) == -2
    assert call(desc(dtype=7)) == -3
    assert call(desc(), ODD) == -4


def test_layer_prefill_workspace_and_argument_checks():
    lib = lisa.library()
    d = lisa.make_desc(lisa.BF16, 2, 32, 8, 256, 256, 128, 22, 64, write_scores=1)
    sz = C.c_size_t
    q, k, v = sz(), sz(), sz()
    assert lib.lisa_layer_offsets(C.byref(d), C.byref(q), C.byref(k), C.byref(v)) == 0
    pre = lisa.workspace_bytes(d, lisa.WS_PREFILL)
    assert q.value >= pre and q.value % 256 == 0
    assert k.value - q.value >= 2 * 32 * 256 * 22 * 2 and v.value - k.value >= 2 * 8 * 256 * 22 * 2
    total = lisa.workspace_bytes(d, lisa.WS_LAYER)
    assert total >= v.value + 2 * 8 * 256 * 128 * 2
    args = [FAKE] * 7
    assert lib.lisa_layer_prefill(C.byref(d), 4096, 1.0e4, *args, FAKE, total - 1, None) == -5
    assert lib.lisa_layer_prefill(C.byref(d), 4096, 1.0e4, None, *args[1:], FAKE, total, None) == -1
    chunk = lisa.make_desc(lisa.BF16, 2, 32, 8, 128, 256, 128, 22, 64)        # Lq != Lk
    assert lib.lisa_layer_prefill(C.byref(chunk), 4096, 1.0e4, *args, FAKE, 1 << 40, None) == -2
    assert lisa.workspace_bytes(chunk, lisa.WS_LAYER) == 0


def test_variant_descriptors_are_validated():
    ok = lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 22, 64, act=lisa.ACT_SILU)
    assert lisa.supported(ok) == 0
    assert lisa.supported(lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 22, 32, act=lisa.ACT_SINGLE)) == 0
    assert lisa.supported(lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 22, 64, act=lisa.ACT_SINGLE)) == -2
    assert lisa.supported(lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 22, 0, mix=lisa.MIX_PLUS)) == 0
    assert lisa.supported(lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 0, 0, mix=lisa.MIX_PLUS)) == -2
    assert lisa.supported(lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 0, 0, mix=lisa.MIX_SHARE)) == 0
    assert lisa.supported(lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 22, 64, act=3)) == -3
    assert lisa.supported(lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 22, 64, mix=4)) == -3
    lib = lisa.library()
    plus = lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 22, 0, mix=lisa.MIX_PLUS)
    big = 1 << 40
    # the FFN weights may be NULL for LiSA_plus, Q_LR / K_LR may not
    assert lib.lisa_attn_prefill(C.byref(plus), None, FAKE, FAKE, FAKE, None, None, FAKE, None, FAKE, big, None) == -1
    relu = lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 22, 64)
    assert lib.lisa_attn_prefill(C.byref(relu), FAKE, FAKE, FAKE, FAKE, FAKE, None, FAKE, None, FAKE, big, None) == -1


def test_layer_decode_workspace_and_argument_checks():
    lib = lisa.library()
    d = lisa.make_desc(lisa.BF16, 4, 32, 8, 1, 300, 128, 22, 64, write_scores=1, kcache_dim_major=1, Lmax=320)
    dec = lisa.workspace_bytes(d, lisa.WS_DECODE)
    total = lisa.workspace_bytes(d, lisa.WS_LAYER_DECODE)
    assert total >= dec + 4 * 32 * 22 * 2
    args = [FAKE] * 9
    assert lib.lisa_layer_decode(C.byref(d), 4096, 1.0e4, *args, FAKE, total - 1, None) == -5
    assert lib.lisa_layer_decode(C.byref(d), 4096, 1.0e4, FAKE, None, *args[2:], FAKE, total, None) == -1
    full = lisa.make_desc(lisa.BF16, 4, 32, 8, 1, 400, 128, 22, 64, kcache_dim_major=1, Lmax=320)   # Lk > Lmax
    assert lib.lisa_layer_decode(C.byref(full), 4096, 1.0e4, *args, FAKE, 1 << 40, None) == -2
    share = lisa.make_desc(lisa.BF16, 4, 32, 8, 1, 300, 128, 0, 0, mix=lisa.MIX_SHARE, Lmax=320)
    assert lib.lisa_layer_decode(C.byref(share), 4096, 1.0e4, *args, FAKE, 1 << 40, None) == -3


def test_strerror_is_defined_for_every_status():
    lib = lisa.library()
    seen = set()
    for s in range(0, -7, -1):
        msg = lib.lisa_strerror(s).decode()
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 7
    assert lib.lisa_strerror(-99).decode() == "unknown status"


@pytest.mark.parametrize("h,l,dk,r,nS", [(32, 2048, 128, 20, 17), (40, 4096, 128, 20, 26),
                                          (32, 1024, 128, 22, 27)])
def test_size_helpers_equal_the_memory_analysis(h, l, dk, r, nS):
    """Sec. 5.2: a prefill score matrix takes h*l*l*2 bytes, the decode row h*l*2 bytes and the
    K cache shrinks by |S|*h*l*(d_k-r)*2 bytes (per sequence)."""
    pre = lisa.make_desc(lisa.BF16, 1, h, h, l, l, dk, r, 64)
    dec = lisa.make_desc(lisa.BF16, 1, h, h, 1, l, dk, r, 64, Lmax=l)
    assert lisa.scores_bytes(pre) == h * l * l * 2
    assert lisa.scores_bytes(dec) == h * l * 2
    assert lisa.kcache_saved_bytes(pre, nS) == nS * h * l * (dk - r) * 2
    # net prefill saving of the paper turns negative exactly when l > |S| (d_k - r)
    net = lisa.kcache_saved_bytes(pre, nS) - lisa.scores_bytes(pre)
    assert net == h * l * (nS * (dk - r) - l) * 2
    assert (net < 0) == (l > nS * (dk - r))
    # the workspace never exceeds one float32 copy of the score tensor
    assert lisa.workspace_bytes(pre, lisa.WS_PREFILL) <= h * l * l * 4 + 256


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 2, 4, 8)
    with pytest.raises(ValueError, match="GPU tensor"):
        lisa.std_attn_scores(x, x)


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: any other count ends with a message and a non-zero status
    before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        p = subprocess.run([sys.executable, os.path.join(root, "bench.py")] + argv, capture_output=True, text=True,
                           env={**os.environ, **env}, timeout=120)
        assert p.returncode != 0
        assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_sharing_patterns_match_the_printed_table():
    """Counts and proportions of the paper's layer-sharing configurations (Sec. 5.1 table), the
    split of the single-layer models into LiSA and direct-sharing layers, and the rule that a
    sharing layer always has a layer in front of it."""
    from paper_2408_01890_amd import patterns
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "sharing_patterns.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 12
    for name, total, sharing, pct in rows:
        p = patterns.PATTERNS[name]
        assert len(p) == int(total) and patterns.sharing_layers(p) == int(sharing)
        assert f"{100.0 * int(sharing) / int(total) + 1e-9:.2f}" == pct
        assert p[0] == patterns.STD and p[1] == patterns.STD and p[2] == patterns.STD
    sl = patterns.PATTERNS["lisa_sl_7_10_of_32"]
    assert (sl.count(patterns.LISA), sl.count(patterns.SHARE)) == (7, 10)        # "LiSA_SL (7+10)"
    sl = patterns.PATTERNS["lisa_sl_10_12_of_40"]
    assert (sl.count(patterns.LISA), sl.count(patterns.SHARE)) == (10, 12)       # "LiSA_SL (10+12)"
    # LiSA (27) shares in 27 consecutive layers, numbers 4..30 (1-based)
    p = patterns.PATTERNS["lisa_27_of_32"]
    assert all(k == patterns.LISA for k in p[3:30]) and p[30] == patterns.STD and p[31] == patterns.STD
    # the sharing layers of a LiSA model and of the DS model of the same size coincide
    for a, b in (("lisa_17_of_32", "ds_17_of_32"), ("lisa_21_of_32", "ds_21_of_32"), ("lisa_26_of_40", "ds_26_of_40")):
        assert [k != patterns.STD for k in patterns.PATTERNS[a]] == [k != patterns.STD for k in patterns.PATTERNS[b]]


def test_decode_stack_rejects_bad_stacks_before_any_launch():
    lib = lisa.library()
    d = lisa.make_desc(lisa.BF16, 2, 8, 4, 1, 100, 128, 22, 32, kcache_dim_major=1, Lmax=128)
    assert lisa.stack_workspace_bytes(d) > 2 * 2 * 8 * 100 * 2
    P = [C.c_void_p(0x10000 + 0x100 * i) for i in range(8)]

    def layer(kind, **kw):
        f = dict(q=P[0], k_cache=P[1], v_cache=P[2], w1=P[3], w2=P[4], out=P[5], score_row=None)
        f.update(kw)
        return lisa.StackLayer(kind, 0, f["q"], f["k_cache"], f["v_cache"], f["w1"], f["w2"], f["out"], f["score_row"])

    def call(layers, ws=P[6], wsb=1 << 40, desc=d):
        arr = (lisa.StackLayer * len(layers))(*layers)
        return lib.lisa_decode_stack(C.byref(desc), arr, len(layers), ws, wsb, None)

    assert call([layer(lisa.LAYER_LISA)]) == -2                             # no front layer to share with
    assert call([layer(lisa.LAYER_STD), layer(7)]) == -2                    # unknown kind
    assert call([layer(lisa.LAYER_STD), layer(lisa.LAYER_LISA, w1=None)]) == -1
    assert call([layer(lisa.LAYER_STD, v_cache=None)]) == -1
    assert call([layer(lisa.LAYER_STD), layer(lisa.LAYER_SHARE, out=ODD)]) == -4
    assert call([layer(lisa.LAYER_STD)], ws=None) == -5
    assert call([layer(lisa.LAYER_STD)], wsb=64) == -5
    assert lib.lisa_decode_stack(C.byref(d), None, 1, P[6], 1 << 40, None) == -1
    bad = lisa.make_desc(lisa.BF16, 2, 8, 4, 1, 100, 128, 22, 32, mix=lisa.MIX_SHARE, kcache_dim_major=1, Lmax=128)
    assert call([layer(lisa.LAYER_STD)], desc=bad) == -2


def test_tiled_score_layout_is_validated_and_sized_on_the_host():
    """score_tiled: a flag of the prefill calls of the bf16 matrix-core kernels (tiles of 16 rows x 32
    keys, 1 KB each); sizes count whole tiles; other values, decode steps and shapes outside those
    kernels are refused before any HIP call."""
    lib = lisa.library()
    d = lisa.make_desc(lisa.BF16, 2, 32, 8, 100, 200, 128, 22, 64, write_scores=1, score_tiled=1)
    assert lib.lisa_scores_elems(C.byref(d)) == 2 * 32 * 7 * 7 * 512          # ceil(100/16) x ceil(200/32) tiles
    assert lisa.scores_bytes(d) == 2 * 32 * 7 * 7 * 512 * 2
    rm = lisa.make_desc(lisa.BF16, 2, 32, 8, 100, 200, 128, 22, 64, write_scores=1)
    assert lib.lisa_scores_elems(C.byref(rm)) == 2 * 32 * 100 * 200
    assert lisa.scores_shape(2, 32, 100, 200, True) == (2, 7, 7, 32, 16, 32)
    assert lib.lisa_scores_elems(None) == 0
    big = 1 << 40
    bad = lisa.make_desc(lisa.BF16, 2, 32, 8, 100, 200, 128, 22, 64, write_scores=1, score_tiled=2)
    assert lib.lisa_attn_prefill(C.byref(bad), *([FAKE] * 6), FAKE, C.c_void_p(0x20000), FAKE, big, None) == -2
    # a decode step hands over score rows, not tiles
    dec = lisa.make_desc(lisa.BF16, 2, 32, 8, 1, 200, 128, 22, 64, write_scores=1, Lmax=256, score_tiled=1)
    ptrs = [C.c_void_p(0x10000 + 0x1000 * i) for i in range(11)]
    assert lib.lisa_attn_decode(C.byref(dec), *ptrs, big, None) == -3
    # shapes whose kernels take row-major scores only (fp32; F beyond the fused kernel; the CONCAT form
    # beyond 32 heads)
    f32 = lisa.make_desc(lisa.F32, 1, 4, 4, 64, 64, 64, 8, 16, write_scores=1, score_tiled=1)
    wide = lisa.make_desc(lisa.BF16, 1, 32, 32, 64, 64, 128, 20, 256, write_scores=1, score_tiled=1)
    cat = lisa.make_desc(lisa.BF16, 1, 40, 40, 64, 64, 128, 20, 256, mix=lisa.MIX_CONCAT, write_scores=1,
                         score_tiled=1)
    for desc in (f32, wide, cat):
        assert lib.lisa_attn_prefill(C.byref(desc), *([FAKE] * 6), FAKE, C.c_void_p(0x20000), FAKE, big, None) == -3
    assert lib.std_attn_scores(C.byref(f32), FAKE, FAKE, None, FAKE, None, None, 0, None) == -3


def test_kd_huber_rejects_bad_arguments_before_any_launch():
    lib = lisa.library()
    d = lisa.make_desc(lisa.BF16, 2, 8, 8, 64, 64, 1)
    need = lisa.workspace_bytes(d, lisa.WS_KD)
    assert need == min((2 * 8 * 64 + 3) // 4, 2048) * 8
    out = C.c_void_p(0x30000)
    assert lib.lisa_kd_huber(C.byref(d), None, FAKE, 1.0, 1.0, 0, out, FAKE, need, None) == -1
    assert lib.lisa_kd_huber(C.byref(d), FAKE, FAKE, 0.0, 1.0, 0, out, FAKE, need, None) == -2
    assert lib.lisa_kd_huber(C.byref(d), FAKE, FAKE, 1.0, float("inf"), 0, out, FAKE, need, None) == -2
    assert lib.lisa_kd_huber(C.byref(d), FAKE, FAKE, 1.0, 1.0, 2, out, FAKE, need, None) == -2
    assert lib.lisa_kd_huber(C.byref(d), FAKE, ODD, 1.0, 1.0, 0, out, FAKE, need, None) == -4
    assert lib.lisa_kd_huber(C.byref(d), FAKE, FAKE, 1.0, 1.0, 0, out, FAKE, need - 1, None) == -5
    assert lib.lisa_kd_huber(C.byref(d), FAKE, FAKE, 1.0, 1.0, 0, out, None, 0, None) == -5
    f32t = lisa.make_desc(lisa.F32, 2, 8, 8, 64, 64, 1, score_tiled=1)
    assert lib.lisa_kd_huber(C.byref(f32t), FAKE, FAKE, 1.0, 1.0, 0, out, FAKE, 1 << 20, None) == -3


def test_reference_kernels_reject_bad_arguments_before_any_launch():
    lib = lisa.library()
    assert lib.lisa_probe_hbm_read(None, 1 << 20, FAKE, None) == -1
    assert lib.lisa_probe_hbm_read(FAKE, 1 << 20, None, None) == -1
    assert lib.lisa_probe_hbm_read(ODD, 1 << 20, FAKE, None) == -4
    assert lib.lisa_probe_hbm_read(FAKE, 8, FAKE, None) == -2
    assert lib.lisa_probe_hbm_write(None, 1 << 20, 1, None) == -1
    assert lib.lisa_probe_hbm_write(ODD, 1 << 20, 1, None) == -4
    assert lib.lisa_probe_hbm_write(FAKE, 15, 1, None) == -2
    assert lib.lisa_probe_mfma(0, 10, 16, None, None) == -1
    assert lib.lisa_probe_mfma(0, 0, 16, FAKE, None) == -2
    assert lib.lisa_probe_mfma(1, 10, 1 << 20, FAKE, None) == -2
