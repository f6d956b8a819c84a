"""GPU parity of harp_grad_blocks (gradient through Y = X U with respect to the blocks and X)
against the float64 oracle, through the C ABI."""
import sys

import numpy as np
import pytest

from oracle import harp_oracle as ho
from paper_2605_29843_amd import inputs as gi
from parity_util import assert_parity, summand_magnitude, to_device, to_host64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def harp():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_29843_amd import harp as h
    return h


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def assert_dk_parity(dK, ref, X, G, what):
    """dK is a float32 sum of n products of float32 numbers.  Per entry the oracle's value is
    bounded by sqrt(sum x^2 sum g^2) <= ||X||_max-col ||G||_max-col; the float32 path (one rounding
    per product and per partial sum, chunks of <= 32..n/128 rows, then <= 128 chunk sums) stays
    within 2e-5 of that scale for the n used here, and must be finite.  With non-orthogonal blocks
    the inner activations x_t and gradients g_t are no longer of the size of X and G; the largest
    entry of the stage's own reference then joins the scale."""
    scale = float(np.sqrt((X.astype(np.float64) ** 2).sum(axis=0).max() *
                          (G.astype(np.float64) ** 2).sum(axis=0).max()))
    for t, (a, r) in enumerate(zip(dK, ref)):
        a = a.detach().cpu().numpy().astype(np.float64)
        assert a.shape == r.shape, (a.shape, r.shape)
        assert np.all(np.isfinite(a))
        err = np.abs(a - r)
        tol = 2e-5 * max(scale, float(np.abs(r).max())) + 1e-5 * np.abs(r)
        assert np.all(err <= tol), f"{what}: stage {t}: max err {err.max():.3e} vs tol {tol.min():.3e}"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,radices,n,kind", [
    (256, [2] * 8, 64, "orth"), (240, [5, 6, 8], 37, "orth"), (96, [3, 2, 2, 2, 4], 1, "generic"),
    (1024, [8, 8, 4, 4], 200, "orth"), (672, [7, 2, 2, 2, 2, 2, 3], 33, "generic"),
    (4096, [2] * 12, 130, "orth"),
    # a stage of radix above 8 (leftover prime): first, last, in the middle, with signs on it
    (44, [4, 11], 9, "generic"), (344, [2, 2, 2, 43], 70, "orth"), (572, [13, 4, 11], 21, "generic"),
    (1376, [2] * 5 + [43], 130, "orth"), (128, [2, 64], 5, "generic"),
    # ... at a stride that is a multiple of 16, in the middle: the stage and the gradient passed
    # back through it both run on the matrix cores
    (704, [4, 4, 11, 2, 2], 50, "generic"), (1408, [2] * 4 + [11, 8], 33, "orth"),
    (320, [4, 4, 20], 75, "generic"), (1024, [2, 2, 2, 2, 64], 12, "orth")])
def test_grad_blocks_matches_the_oracle(harp, d, radices, n, kind, dtype):
    import torch
    rng = np.random.default_rng(d + n)
    blocks = gi.make_blocks(d, radices, kind, rng)
    signs = gi.make_signs(d, rng)
    X = rng.standard_normal((n, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    if dtype == "bf16":
        X, G = gi.round_to_bf16(X), gi.round_to_bf16(G)
    plan = harp.Plan(d, radices, blocks, signs)
    say("grad_blocks", d, radices, n, kind, dtype)
    dK, dX = harp.harp_grad_blocks(plan, to_device(X, dtype), to_device(G, dtype))
    torch.cuda.synchronize()
    rK, rX = ho.grad_blocks(X, G, d, radices, blocks, signs)
    assert_dk_parity(dK, rK, X, G, "dK")
    mag = None
    if kind == "generic":    # the blocks really are non-orthogonal, and the tolerance follows the summands
        assert max(float(np.abs(np.swapaxes(K, 1, 2) @ K - np.eye(K.shape[1])).max()) for K in blocks) > 0.05
        mag = summand_magnitude(G, d, radices, blocks, transpose=True)
    assert_parity(to_host64(dX), rX, dtype, "dX", mag=mag)
    # dX is apply_transpose of G
    Z = harp.harp_apply_transpose(plan, to_device(G, dtype))
    assert_parity(to_host64(Z), rX, dtype, "apply_transpose(G)", mag=mag)
    # the same call again gives the same bits (fixed summation order)
    dK2, _ = harp.harp_grad_blocks(plan, to_device(X, dtype), to_device(G, dtype), want_dX=False)
    torch.cuda.synchronize()
    for a, b in zip(dK, dK2):
        assert torch.equal(a, b)
    plan.destroy()


def test_grad_blocks_without_signs_and_with_padded_rows(harp):
    import torch
    d, radices, n = 512, [2, 4, 8, 8], 70
    rng = np.random.default_rng(9)
    blocks = gi.make_blocks(d, radices, "orth", rng)
    X = rng.standard_normal((n, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    plan = harp.Plan(d, radices, blocks, None)
    bigx = torch.zeros(n, d + 24, device="cuda")
    bigg = torch.zeros(n, d + 8, device="cuda")
    bigx[:, 3:3 + d] = torch.from_numpy(X).cuda()
    bigg[:, 5:5 + d] = torch.from_numpy(G).cuda()
    dK, dX = harp.harp_grad_blocks(plan, bigx[:, 3:3 + d], bigg[:, 5:5 + d])
    torch.cuda.synchronize()
    rK, rX = ho.grad_blocks(X, G, d, radices, blocks, None)
    assert_dk_parity(dK, rK, X, G, "dK (views)")
    assert_parity(to_host64(dX), rX, "f32", "dX (views)")
    plan.destroy()


def test_grad_blocks_empty_batch(harp):
    import torch
    d, radices = 64, [4, 4, 4]
    rng = np.random.default_rng(1)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng), gi.make_signs(d, rng))
    X = torch.empty(0, d, device="cuda")
    dK, dX = harp.harp_grad_blocks(plan, X, X.clone())
    torch.cuda.synchronize()
    assert all(float(k.abs().max()) == 0.0 for k in dK) and dX.shape == (0, d)
    plan.destroy()


def test_grad_blocks_llama7b_shape_sampled(harp):
    """2048 x 4096 bf16, 12 radix-2 stages (the benchmark's shape): every block of every stage
    against the oracle on the same rows."""
    import torch
    w = gi.workload("llama7b_4096_r2")
    d, radices, n = w["d"], w["radices"], w["n"]
    rng = np.random.default_rng(4)
    X = w["X"]
    G = gi.round_to_bf16((rng.standard_normal((n, d)) * 0.05).astype(np.float32))
    plan = harp.Plan(d, radices, w["blocks"], w["signs"])
    say("grad_blocks full size", n, d)
    dK, dX = harp.harp_grad_blocks(plan, to_device(X, "bf16"), to_device(G, "bf16"))
    torch.cuda.synchronize()
    rK, rX = ho.grad_blocks(X, G, d, radices, w["blocks"], w["signs"])
    assert_dk_parity(dK, rK, X, G, "dK full size")
    rows = np.arange(0, n, 97)
    assert_parity(to_host64(dX)[rows], rX[rows], "bf16", "dX rows")
    plan.destroy()
