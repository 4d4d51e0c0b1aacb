"""Seeded synthetic workloads shaped like the paper's LLaMA layers.

This module only *draws and prepares inputs*; it contains none of the LiSA layer's
arithmetic (no scores, no alignment FFN, no softmax).  Both the HIP library and the CPU
oracle are fed the arrays produced here, already rounded to the configuration's dtype.

Recipe (stands in for the trained LLaMA2-7B / LLaMA3-8B / LLaMA2-13B layers of Sec. 5.3
and App. C.1, whose weights are not available): hidden states X ~ N(0,1); projection and FFN
weights ~ N(0, 0.02^2); Q_LR = X W^Q_LR, K_LR = X W^K_LR, V = X W^V by one library matmul
(input preparation outside the library boundary; Eq. 3's `H W_LR` factor); optional rotary
position embedding on Q_LR / K_LR (over r) and on the standard layer's Q / K (over d_k); the
standard layer's Q, K ~ N(0,1).  Everything is rounded once to the dtype.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import torch


@dataclasses.dataclass(frozen=True)
class LayerShape:
    name: str
    dtype: str                 # "f32" | "bf16"
    B: int
    H: int
    Hkv: int
    L: int
    d_model: int
    d_k: int
    r: int
    F: int
    rope_theta: Optional[float] = None

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def score_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.float16

    def scaled(self, **kw) -> "LayerShape":
        return dataclasses.replace(self, **kw)


# The four prefill configurations and the decode stack of the benchmark definition.
C1 = LayerShape("c1_f32_l128", "f32", 1, 8, 8, 128, 512, 64, 11, 32)
C2 = LayerShape("c2_llama2_7b_l2048", "bf16", 1, 32, 32, 2048, 4096, 128, 22, 64)
C3 = LayerShape("c3_llama3_8b_gqa_l8192", "bf16", 4, 32, 8, 8192, 4096, 128, 22, 64, 500000.0)
C4 = LayerShape("c4_llama2_13b_l4096", "bf16", 8, 40, 40, 4096, 5120, 128, 22, 80)
PREFILL_CONFIGS = {c.name: c for c in (C1, C2, C3, C4)}


@dataclasses.dataclass(frozen=True)
class DecodeStack:
    name: str
    dtype: str
    B: int
    H: int
    Hkv: int
    ctx: int                   # cached tokens before the step; the step attends ctx + 1 keys
    d_model: int
    d_k: int
    r: int
    F: int
    n_layers: int
    n_std: int                 # layers 0 .. n_std-1 are standard attention, the rest LiSA

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def score_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.float16

    def scaled(self, **kw) -> "DecodeStack":
        return dataclasses.replace(self, **kw)


C5 = DecodeStack("c5_llama2_7b_decode_ctx4096", "bf16", 64, 32, 32, 4096, 4096, 128, 22, 64, 32, 5)

BASE_SEED = 20240801


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, g, device, std=1.0):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std


def rope_(x: torch.Tensor, theta: float, pos0: int = 0) -> torch.Tensor:
    """Rotary embedding over the last axis of x [..., L, n] (n even), half-split pairing
    (t, t + n/2), angle = pos * theta^(-2t/n).  Input preparation, float64 internally."""
    n = x.shape[-1]
    assert n % 2 == 0, "rotary embedding needs an even width"
    L = x.shape[-2]
    half = n // 2
    pos = torch.arange(pos0, pos0 + L, device=x.device, dtype=torch.float64)[:, None]
    inv = theta ** (-torch.arange(0, half, device=x.device, dtype=torch.float64) * 2.0 / n)[None, :]
    ang = pos * inv
    c, s = torch.cos(ang), torch.sin(ang)
    xd = x.double()
    a, b = xd[..., :half], xd[..., half:]
    return torch.cat([a * c - b * s, a * s + b * c], dim=-1).to(x.dtype)


def ffn_weights(H: int, F: int, mix: str, kind: str, g, device, dtype):
    """W1 [Din,F], W2 [F,H].  kind: 'paper' N(0,0.02^2) | 'fan_in' N(0,1/fan_in) |
    'identity_noise' ([I,-I] / [I;-I] acting on A_{n-1}, plus N(0,0.02^2); needs F >= 2H)."""
    Din = 2 * H if mix == "concat" else H
    if kind == "paper":
        w1 = _randn((Din, F), g, device, 0.02)
        w2 = _randn((F, H), g, device, 0.02)
    elif kind == "fan_in":
        w1 = _randn((Din, F), g, device, 1.0 / math.sqrt(Din))
        w2 = _randn((F, H), g, device, 1.0 / math.sqrt(F))
    elif kind == "identity_noise":
        assert F >= 2 * H, "identity through ReLU needs F >= 2H"
        w1 = _randn((Din, F), g, device, 0.02)
        w2 = _randn((F, H), g, device, 0.02)
        eye = torch.eye(H, device=device)
        w1[:H, :H] += eye
        w1[:H, H:2 * H] -= eye
        w2[:H, :] += eye
        w2[H:2 * H, :] -= eye
    else:
        raise ValueError(kind)
    return w1.to(dtype).contiguous(), w2.to(dtype).contiguous()


def _project(x, w, heads, width):
    """[B,L,d] @ [d, heads*width] -> [B,heads,L,width] (float32 library matmul)."""
    B, L, _ = x.shape
    y = x @ w
    return y.view(B, L, heads, width).permute(0, 2, 1, 3).contiguous()


def make_prefill_inputs(cfg: LayerShape, seed: int = BASE_SEED, device="cpu", mix: str = "add",
                        ffn: str = "paper", std_layer: bool = True) -> Dict[str, torch.Tensor]:
    """Inputs of one LiSA prefill layer (+ the Q, K of the standard layer that feeds it).

    Returns tensors in cfg dtype: q_lr [B,H,L,r], k_lr [B,Hkv,L,r], v [B,Hkv,L,d_k],
    w1, w2, and (std_layer) q [B,H,L,d_k], k [B,Hkv,L,d_k].
    """
    g = _gen(seed, device)
    dt = cfg.torch_dtype
    out: Dict[str, torch.Tensor] = {}
    x = _randn((cfg.B, cfg.L, cfg.d_model), g, device)
    wq = _randn((cfg.d_model, cfg.H * cfg.r), g, device, 0.02)
    wk = _randn((cfg.d_model, cfg.Hkv * cfg.r), g, device, 0.02)
    wv = _randn((cfg.d_model, cfg.Hkv * cfg.d_k), g, device, 0.02)
    q_lr = _project(x, wq, cfg.H, cfg.r)
    k_lr = _project(x, wk, cfg.Hkv, cfg.r)
    v = _project(x, wv, cfg.Hkv, cfg.d_k)
    del x, wq, wk, wv
    if cfg.rope_theta is not None:
        q_lr = rope_(q_lr, cfg.rope_theta)
        k_lr = rope_(k_lr, cfg.rope_theta)
    out["q_lr"], out["k_lr"], out["v"] = q_lr.to(dt), k_lr.to(dt), v.to(dt)
    out["w1"], out["w2"] = ffn_weights(cfg.H, cfg.F, mix, ffn, g, device, dt)
    if std_layer:
        q = _randn((cfg.B, cfg.H, cfg.L, cfg.d_k), g, device)
        k = _randn((cfg.B, cfg.Hkv, cfg.L, cfg.d_k), g, device)
        if cfg.rope_theta is not None:
            q = rope_(q, cfg.rope_theta)
            k = rope_(k, cfg.rope_theta)
        out["q"], out["k"] = q.to(dt), k.to(dt)
    return out


def make_projection_inputs(cfg: LayerShape, seed: int = BASE_SEED + 9, device="cpu",
                           L: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """Operands of the projection front end: hidden states x [B,L,d_model] ~ N(0,1) and the
    stacked weight rows w [H*r + Hkv*r + Hkv*d_k, d_model] ~ N(0, 0.02^2) (W^Q_LR, W^K_LR, W^V,
    one row per output feature), rounded to cfg dtype.  Draws only; no product is formed here."""
    g = _gen(seed, device)
    dt = cfg.torch_dtype
    L = cfg.L if L is None else L
    x = _randn((cfg.B, L, cfg.d_model), g, device).to(dt)
    n = (cfg.H + cfg.Hkv) * cfg.r + cfg.Hkv * cfg.d_k
    w = _randn((n, cfg.d_model), g, device, 0.02).to(dt)
    return {"x": x.contiguous(), "w": w.contiguous()}


def make_decode_layer(stk: DecodeStack, layer: int, seed: int = BASE_SEED + 5, device="cpu",
                      mix: str = "add", ffn: str = "paper", dim_major: bool = True,
                      Lmax: Optional[int] = None, kind: Optional[str] = None) -> Dict[str, torch.Tensor]:
    """Caches and the new token's projections of one layer of the decode stack.

    Caches are filled with N(0,1) values up to and including the new token (index ctx), so
    the step needs no append; `k_lr_new` / `v_new` are also returned (equal to the cache
    entries at index ctx) for callers that exercise the append path.
    Standard layers (layer < n_std): q [B,H,d_k], k_cache [B,Hkv,Lmax,d_k], v_cache.
    LiSA layers: q_lr [B,H,r], k_lr_cache ([B,Hkv,r,Lmax] if dim_major else [B,Hkv,Lmax,r]),
    v_cache [B,Hkv,Lmax,d_k], w1, w2.
    kind: "std" | "lisa" | "share" overrides the stack's own split (layer < n_std is standard);
    a direct-sharing layer ("share") has a V cache only.
    """
    g = _gen(seed * 1000 + layer, device)
    dt = stk.torch_dtype
    Lk = stk.ctx + 1
    Lmax = Lk if Lmax is None else Lmax
    assert Lmax >= Lk
    out: Dict[str, torch.Tensor] = {}

    def cache(width):
        c = torch.zeros((stk.B, stk.Hkv, Lmax, width), device=device, dtype=dt)
        c[:, :, :Lk] = _randn((stk.B, stk.Hkv, Lk, width), g, device).to(dt)
        return c

    out["v_cache"] = cache(stk.d_k)
    out["v_new"] = out["v_cache"][:, :, Lk - 1].contiguous()
    if kind is None:
        kind = "std" if layer < stk.n_std else "lisa"
    if kind == "share":
        return out
    if kind == "std":
        out["q"] = _randn((stk.B, stk.H, stk.d_k), g, device).to(dt)
        out["k_cache"] = cache(stk.d_k)
    else:
        out["q_lr"] = _randn((stk.B, stk.H, stk.r), g, device).to(dt)
        kc = cache(stk.r)
        out["k_lr_new"] = kc[:, :, Lk - 1].contiguous()
        out["k_lr_cache"] = kc.permute(0, 1, 3, 2).contiguous() if dim_major else kc
        out["w1"], out["w2"] = ffn_weights(stk.H, stk.F, mix, ffn, g, device, dt)
    return out


def sample_rows(L: int, n: int, seed: int, tile: int = 64):
    """Row indices for sampled parity: first rows, last row, tile-boundary rows +-1 and
    uniformly drawn rows; sorted, unique."""
    g = torch.Generator().manual_seed(int(seed))
    rows = {0, 1, 2, L - 1, L - 2}
    for t in (tile, 2 * tile, L // 2, L - tile):
        for d in (-1, 0, 1):
            if 0 <= t + d < L:
                rows.add(t + d)
    extra = torch.randint(0, L, (max(n - len(rows), 0),), generator=g).tolist()
    rows.update(extra)
    return sorted(r for r in rows if 0 <= r < L)
