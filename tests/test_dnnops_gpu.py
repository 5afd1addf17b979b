"""Parity of the Mish / layer-normalisation / softmax kernels (through the C ABI) against the
fp64 CPU oracle.  fp32 tolerances: 1e-4 forward, 1e-3 gradients, element by element relative
to max(|ref_i|, rms(ref))."""
import numpy as np
import pytest

from oracle import dnnops as orc
from parity_util import rel_err

pytestmark = pytest.mark.gpu
FWD, GRAD = 1e-4, 1e-3


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0")


def _host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("n", [1, 3, 4, 1027, 8 * 1024 * 1024 + 5])
def test_mish_matches_oracle(n):
    import torch
    from paper_2110_10802_amd import dnnops as D
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * 4).astype(np.float32)
    if n >= 1027:  # the tails of the function: saturation on both sides and the overflow guard
        x[:8] = [-100.0, -30.0, -12.0, 0.0, 12.0, 19.99, 25.0, 90.0]
    dy = rng.standard_normal(n).astype(np.float32)
    xd, dyd = _dev(x), _dev(dy)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    print(f"[dnnops] mish n={n}", flush=True)
    D.mish_forward(xd, y, n)
    D.mish_backward(xd, dyd, dx, n)
    torch.cuda.synchronize()
    assert rel_err(_host(y), orc.mish_fwd(x)) <= FWD
    assert rel_err(_host(dx), orc.mish_bwd(x, dy)) <= GRAD


ROW_SHAPES = [(1, 4), (3, 8), (5, 252), (7, 256), (4096, 1024), (33, 2048), (9, 1), (6, 37),
              (11, 2052), (3, 8192)]


def _random_rows(count, seed):
    """Seeded random (rows, cols): row lengths log-uniform from 1 to 9000, so every row-kernel
    variant and its ragged tail is reached."""
    import random
    rng = random.Random(seed)
    return [(rng.randint(1, 200), max(1, int(round(9000 ** rng.random())))) for _ in range(count)]


ROW_SHAPES += _random_rows(24, seed=20211020)


@pytest.mark.parametrize("rows,cols", ROW_SHAPES)
def test_layernorm_matches_oracle(rows, cols):
    import torch
    from paper_2110_10802_amd import dnnops as D
    rng = np.random.default_rng(rows * 100003 + cols)
    x = (rng.standard_normal((rows, cols)) * 2 + 0.5).astype(np.float32)
    gamma = (1 + 0.1 * rng.standard_normal(cols)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(cols)).astype(np.float32)
    dy = rng.standard_normal((rows, cols)).astype(np.float32)
    eps = 1e-5
    xd, gd, bd, dyd = _dev(x), _dev(gamma), _dev(beta), _dev(dy)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    mean = torch.empty(rows, device="cuda:0")
    rstd = torch.empty(rows, device="cuda:0")
    dg, db = torch.empty_like(gd), torch.empty_like(gd)
    scratch = torch.empty(max(D.layernorm_backward_scratch_bytes(rows, cols), 16),
                          dtype=torch.uint8, device="cuda:0")
    print(f"[dnnops] layernorm {rows}x{cols}", flush=True)
    D.layernorm_forward(xd, gd, bd, eps, rows, cols, y, mean, rstd)
    D.layernorm_backward(xd, dyd, gd, mean, rstd, rows, cols, dx, dg, db, scratch)
    torch.cuda.synchronize()
    yo, mo, ro = orc.layernorm_fwd(x, gamma, beta, eps)
    assert rel_err(_host(y), yo) <= FWD
    assert rel_err(_host(mean), mo) <= FWD and rel_err(_host(rstd), ro) <= FWD
    dxo, dgo, dbo = orc.layernorm_bwd(x, dy, gamma, mo, ro)
    # dx is rstd times a difference of terms of size |dy*gamma| that cancels completely for very
    # short rows (cols = 1: dx = 0 exactly), so the error is measured against the size of those
    # terms; for ordinary rows that is the tensor's own rms
    scale = float(np.sqrt(np.mean((dy.astype(np.float64) * gamma) ** 2)) * np.max(ro))
    assert rel_err(_host(dx), dxo, abs_floor=scale) <= GRAD
    xh_rms = float(np.sqrt(np.mean(((x - mo[:, None]) * ro[:, None]) ** 2)))
    gfloor = float(np.sqrt(np.mean(dy.astype(np.float64) ** 2)) * np.sqrt(rows)) * max(xh_rms, 1e-30)
    assert rel_err(_host(dg), dgo, abs_floor=gfloor) <= GRAD and rel_err(_host(db), dbo) <= GRAD
    # bitwise repeatable (fixed-order reductions)
    dg2, db2 = torch.empty_like(dg), torch.empty_like(db)
    D.layernorm_backward(xd, dyd, gd, mean, rstd, rows, cols, dx, dg2, db2, scratch)
    torch.cuda.synchronize()
    assert torch.equal(dg, dg2) and torch.equal(db, db2)


@pytest.mark.parametrize("rows,cols", ROW_SHAPES + [(8 * 16 * 512, 512)])
def test_softmax_matches_oracle(rows, cols):
    import torch
    from paper_2110_10802_amd import dnnops as D
    rng = np.random.default_rng(rows * 7919 + cols)
    x = (rng.standard_normal((rows, cols)) * 3).astype(np.float32)
    x[0, 0] = 80.0  # a dominant entry: exp must not overflow
    dy = rng.standard_normal((rows, cols)).astype(np.float32)
    xd, dyd = _dev(x), _dev(dy)
    y, dx = torch.empty_like(xd), torch.empty_like(xd)
    print(f"[dnnops] softmax {rows}x{cols}", flush=True)
    D.softmax_forward(xd, y, rows, cols)
    D.softmax_backward(y, dyd, dx, rows, cols)
    torch.cuda.synchronize()
    yo = orc.softmax_fwd(x)
    yh = _host(y)
    assert rel_err(yh, yo) <= FWD
    assert np.allclose(yh.sum(axis=1), 1.0, atol=1e-5)
    # backward is checked on the GPU's own y (the value the call was given)
    assert rel_err(_host(dx), orc.softmax_bwd(yh, dy)) <= GRAD
