"""The no-allocation entry point (dnnops_layernorm_backward_noalloc, for callers that cannot
allocate device memory: HIP graph capture, tight serving loops) against the existing entry
point it is a variant of, through the C ABI: two calls in a row on one GPU, the second with a
smaller input, so that the library's static scratch buffer still holds the first call's
partial sums when the second runs.  Same kernels and the same fixed summation order, so the
results must agree bit for bit; both are also held to the oracle at the gradient tolerance."""
import numpy as np
import pytest

from oracle import dnnops as orc
from parity_util import rel_err

pytestmark = pytest.mark.gpu
GRAD = 1e-3


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0")


def _host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _case(rows, cols):
    rng = np.random.default_rng(rows * 7919 + cols)
    x = (rng.standard_normal((rows, cols)) * 2 + 0.5).astype(np.float32)
    gamma = (1 + 0.1 * rng.standard_normal(cols)).astype(np.float32)
    beta = (0.1 * rng.standard_normal(cols)).astype(np.float32)
    dy = rng.standard_normal((rows, cols)).astype(np.float32)
    return x, gamma, beta, dy


# (first call, second smaller call): rows in registers (cols % 4 == 0, <= 2048), then the
# row-in-LDS path with its column-sum kernel (a row length that is not a multiple of four)
@pytest.mark.parametrize("first,second", [((4096, 1024), (37, 300)), ((700, 2050), (50, 771)),
                                          ((900, 2048), (3, 1030))])
def test_noalloc_matches_the_workspace_entry_point_twice_in_a_row(first, second):
    import torch
    from paper_2110_10802_amd import dnnops as D

    eps = 1e-5
    prepared = []
    for rows, cols in (first, second):
        x, gamma, beta, dy = _case(rows, cols)
        xd, gd, bd, dyd = _dev(x), _dev(gamma), _dev(beta), _dev(dy)
        y = torch.empty_like(xd)
        mean, rstd = torch.empty(rows, device="cuda:0"), torch.empty(rows, device="cuda:0")
        D.layernorm_forward(xd, gd, bd, eps, rows, cols, y, mean, rstd)
        need = D.layernorm_backward_scratch_bytes(rows, cols)
        assert 0 < need <= D.layernorm_backward_noalloc_max_scratch_bytes()
        scratch = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        ref = [torch.empty_like(xd), torch.empty_like(gd), torch.empty_like(gd)]
        D.layernorm_backward(xd, dyd, gd, mean, rstd, rows, cols, *ref, scratch)
        got = [torch.full_like(xd, float("nan")), torch.full_like(gd, float("nan")),
               torch.full_like(gd, float("nan"))]
        prepared.append((rows, cols, x, gamma, beta, dy, xd, gd, dyd, mean, rstd, ref, got))
    torch.cuda.synchronize()
    # the two calls under test, back to back: nothing is allocated between or inside them
    for rows, cols, _, _, _, _, xd, gd, dyd, mean, rstd, _, got in prepared:
        print(f"[no-alloc] layernorm backward {rows}x{cols}", flush=True)
        D.layernorm_backward_noalloc(xd, dyd, gd, mean, rstd, rows, cols, *got)
    torch.cuda.synchronize()
    for rows, cols, x, gamma, beta, dy, _, _, _, _, _, ref, got in prepared:
        for name, r, g in zip(("dx", "dgamma", "dbeta"), ref, got):
            assert torch.equal(r, g), (rows, cols, name)
        _, mo, ro = orc.layernorm_fwd(x, gamma, beta, eps)
        dxo, dgo, dbo = orc.layernorm_bwd(x, dy, gamma, mo, ro)
        assert rel_err(_host(got[0]), dxo) <= GRAD
        assert rel_err(_host(got[1]), dgo) <= GRAD
        assert rel_err(_host(got[2]), dbo) <= GRAD


def test_noalloc_rejects_what_does_not_fit():
    """A shape whose partial sums exceed the static buffer is refused on the host (no launch)."""
    from paper_2110_10802_amd import dnnops as D
    rows, cols = 100000, 8192
    assert D.layernorm_backward_scratch_bytes(rows, cols) > D.layernorm_backward_noalloc_max_scratch_bytes()
    with pytest.raises(D.DnnOpsError) as exc:
        D.layernorm_backward_noalloc(256, 512, 768, 1024, 1280, rows, cols, 1536, 1792, 2048)
    assert exc.value.status == -3
