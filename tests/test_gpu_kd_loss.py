"""lisa_kd_huber (Sec. 5.1 training strategy, App. C.1 Huber loss) against the float64 oracle."""
import numpy as np
import pytest
import torch

from oracle import npref
from paper_2408_01890_amd import lisa
from tests import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda"
RTOL = 2e-6      # float32 per element and per lane, float64 from the wave sums on


def pair(shape, dtype, seed, spread=2.0):
    g = torch.Generator(device=DEV).manual_seed(seed)
    t = (torch.randn(shape, generator=g, device=DEV) * 3).to(dtype)
    s = (t.float() + torch.randn(shape, generator=g, device=DEV) * spread).to(dtype)   # both regimes of the loss
    return s, t


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("dtype,B,H,Lq,Lk", [(torch.float32, 2, 3, 37, 53), (torch.float16, 2, 5, 70, 72),
                                             (torch.float16, 1, 4, 33, 45), (torch.float16, 3, 8, 200, 200),
                                             (torch.float16, 1, 32, 1, 520)])
def test_kd_huber_row_major(dtype, B, H, Lq, Lk, causal):
    s, t = pair((B, H, Lq, Lk), dtype, 11)
    for delta in (1.0, 0.5):
        out = lisa.lisa_kd_huber(s, t, delta=delta, causal=causal)
        torch.cuda.synchronize()
        want = npref.kd_loss(hp.f64(s), hp.f64(t), delta, causal)
        got = out.cpu().numpy()
        print(f"[parity] kd huber {dtype} B{B}H{H} {Lq}x{Lk} causal={causal} delta={delta}: got {got[1]:.9g} want {want:.9g}",
              flush=True)
        assert abs(got[1] - want) <= RTOL * want and got[0] == got[1]
    assert lisa.last_path() == "kd_huber"


@pytest.mark.parametrize("B,H,Lq,Lk", [(2, 8, 100, 200), (1, 32, 264, 264), (1, 40, 17, 40)])
def test_kd_huber_tiled_equals_row_major_and_the_oracle(B, H, Lq, Lk):
    s, t = pair((B, H, Lq, Lk), torch.float16, 12)
    want = npref.kd_loss(hp.f64(s), hp.f64(t))
    st, tt = lisa.tile_scores(s), lisa.tile_scores(t)
    # what a tile holds above the diagonal or beyond the tensor must not count
    junk = torch.full_like(st, 1000.0)
    vis = torch.ones(Lq, Lk, dtype=torch.bool, device=DEV).tril(Lk - Lq)
    stj = lisa.tile_scores(torch.where(vis, s, torch.full_like(s, 1000.0)))
    stj = torch.where(lisa.tile_scores(torch.ones_like(s)) > 0, stj, junk)          # padding rows / keys
    a = lisa.lisa_kd_huber(s, t).cpu().numpy()
    b = lisa.lisa_kd_huber(st, tt, Lq=Lq, Lk=Lk, tiled=True).cpu().numpy()
    c = lisa.lisa_kd_huber(stj, tt, Lq=Lq, Lk=Lk, tiled=True).cpu().numpy()
    assert abs(a[1] - want) <= RTOL * want and abs(b[1] - want) <= RTOL * want and c[1] == b[1]


def test_kd_huber_accumulates_the_mean_over_the_layers_of_s():
    """L_KD = 1/|S| sum over the layers: |S| calls with weight 1/|S| into one result."""
    n = 3
    out = torch.zeros(2, dtype=torch.float64, device=DEV)
    want = 0.0
    for k in range(n):
        s, t = pair((2, 4, 64, 64), torch.float16, 20 + k, spread=0.5 + k)
        lisa.lisa_kd_huber(s, t, weight=1.0 / n, accumulate=k > 0, out=out)
        want += npref.kd_loss(hp.f64(s), hp.f64(t)) / n
    got = out.cpu().numpy()
    assert abs(got[0] - want) <= 2 * RTOL * want
    # twice the same call gives the same bits (fixed order of the partial sums)
    s, t = pair((2, 4, 64, 64), torch.float16, 31)
    x = lisa.lisa_kd_huber(s, t).cpu().numpy()
    y = lisa.lisa_kd_huber(s, t).cpu().numpy()
    assert x[1] == y[1]


def test_kd_huber_closed_forms_at_the_benchmark_size():
    """LLaMA2-7B shape at L = 2048, tiled: constant differences have closed forms at any size."""
    B, H, L = 1, 32, 2048
    shape = lisa.scores_shape(B, H, L, L, True)
    t = torch.zeros(shape, dtype=torch.float16, device=DEV)
    for diff, want in ((0.25, 0.03125), (4.0, 3.5), (0.0, 0.0)):
        s = torch.full(shape, diff, dtype=torch.float16, device=DEV)
        got = lisa.lisa_kd_huber(s, t, Lq=L, Lk=L, tiled=True).cpu().numpy()[1]
        assert abs(got - want) <= 1e-6 * max(want, 1e-30)


def test_kd_huber_rejects_bad_arguments():
    s, t = pair((1, 2, 16, 16), torch.float16, 1)
    for kw in (dict(delta=0.0), dict(delta=float("nan")), dict(weight=float("inf"))):
        with pytest.raises(lisa.LisaError) as e:
            lisa.lisa_kd_huber(s, t, **kw)
        assert e.value.status == -2
