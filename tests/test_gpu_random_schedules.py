"""Seeded random schedules through every kernel-selection path: apply, apply_transpose, the two-sided
rotation (both directions) and the block gradients against the oracle.  The draws are fixed by
their seeds, so a failure names a reproducible case."""
import sys

import numpy as np
import pytest

from oracle import harp_oracle as ho
from paper_2605_29843_amd import inputs as gi
from parity_util import assert_parity, summand_magnitude, to_device, to_host64

pytestmark = pytest.mark.gpu

SMALL = [2, 2, 2, 2, 3, 4, 5, 6, 7, 8]
ANY = SMALL + [9, 11, 13, 16]


@pytest.fixture(scope="module")
def harp():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_29843_amd import harp as h
    return h


def say(*a):
    print(*a, file=sys.stderr, flush=True)


def draw_schedule(rng, pool, dmax, mmax=9):
    radices, d = [], 1
    while len(radices) < mmax:
        b = int(rng.choice(pool))
        if d * b > dmax:
            break
        radices.append(b)
        d *= b
    if not radices:
        radices, d = [2], 2
    return d, radices


@pytest.mark.parametrize("seed", range(24))
def test_random_schedule_apply_and_transpose(harp, seed):
    import torch
    rng = np.random.default_rng(9000 + seed)
    dmax = int(rng.choice([64, 600, 3000, 9000, 20000]))
    d, radices = draw_schedule(rng, ANY, dmax)
    n = int(rng.choice([1, 2, 7, 33, 130]))
    dtype = "bf16" if seed % 2 else "f32"
    kind = "orth" if seed % 3 else "generic"
    pad = int(rng.choice([0, 0, 3, 8]))
    blocks = gi.make_blocks(d, radices, kind, rng)
    signs = gi.make_signs(d, rng) if seed % 4 else None
    X = rng.standard_normal((n, d)).astype(np.float32)
    if dtype == "bf16":
        X = gi.round_to_bf16(X)
    plan = harp.Plan(d, radices, blocks, signs)
    say(f"random schedule seed={seed} d={d} radices={radices} n={n} {dtype} {kind} pad={pad} "
        f"kernel={plan.kernel_name(n)}")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Xf = torch.zeros((n, d + pad), dtype=tdt, device="cuda")
    Xd = Xf[:, :d]
    Xd.copy_(to_device(X, dtype))
    Yf = torch.full((n, d + pad), 5.0, dtype=tdt, device="cuda")
    Yd = Yf[:, :d]
    # non-orthogonal blocks: float32 rounding is relative to the summands of an output entry
    mag = summand_magnitude(X, d, radices, blocks) if kind == "generic" else None
    magt = summand_magnitude(X, d, radices, blocks, transpose=True) if kind == "generic" else None
    if kind == "generic":
        assert max(float(np.abs(np.swapaxes(K, 1, 2) @ K - np.eye(K.shape[1])).max()) for K in blocks) > 0.05
    harp.harp_apply(plan, Xd, Yd)
    torch.cuda.synchronize()
    assert_parity(to_host64(Yd), ho.apply_staged(X, d, radices, blocks, signs), dtype, "apply", mag=mag)
    harp.harp_apply_transpose(plan, Xd, Yd)
    torch.cuda.synchronize()
    assert_parity(to_host64(Yd), ho.apply_transpose_staged(X, d, radices, blocks, signs), dtype,
                  "apply_transpose", mag=magt)
    if pad:
        assert bool((Yf[:, d:] == 5.0).all()), "padding columns were written"
    # in place
    harp.harp_apply(plan, Xd, Xd)
    torch.cuda.synchronize()
    assert_parity(to_host64(Xd), ho.apply_staged(X, d, radices, blocks, signs), dtype, "apply in place",
                  mag=mag)
    plan.destroy()


@pytest.mark.parametrize("seed", range(12))
def test_random_two_sided_rotation(harp, seed):
    import torch
    rng = np.random.default_rng(7000 + seed)
    do, ru = draw_schedule(rng, SMALL if seed % 4 else ANY, int(rng.choice([40, 300, 1100])))
    di, rv = draw_schedule(rng, ANY, int(rng.choice([60, 500, 6000])))
    dtype = "bf16" if seed % 2 else "f32"
    bu, bv = gi.make_blocks(do, ru, "orth", rng), gi.make_blocks(di, rv, "orth", rng)
    su, sv = gi.make_signs(do, rng), gi.make_signs(di, rng)
    W = rng.standard_normal((do, di)).astype(np.float32)
    if dtype == "bf16":
        W = gi.round_to_bf16(W)
    pu, pv = harp.Plan(do, ru, bu, su), harp.Plan(di, rv, bv, sv)
    say(f"random rotation seed={seed} U {do} {ru}  V {di} {rv} {dtype}")
    Wd = to_device(W, dtype)
    out = harp.harp_rotate_weight(pu, pv, Wd)
    inv = harp.harp_rotate_weight_inverse(pu, pv, Wd)
    torch.cuda.synchronize()
    W64 = W.astype(np.float64)
    Uu = ho.build_U(do, ru, bu, su)
    ref = ho.apply_staged(Uu.T @ W64, di, rv, bv, sv)
    refi = ho.apply_transpose_staged(Uu @ W64, di, rv, bv, sv)
    assert_parity(to_host64(out), ref, dtype, "U^T W V")
    assert_parity(to_host64(inv), refi, dtype, "U W V^T")
    pu.destroy()
    pv.destroy()


@pytest.mark.parametrize("seed", range(8))
def test_random_block_gradients(harp, seed):
    import torch
    rng = np.random.default_rng(5000 + seed)
    d, radices = draw_schedule(rng, SMALL, int(rng.choice([50, 700, 5000])))
    n = int(rng.choice([1, 5, 40, 300]))
    dtype = "bf16" if seed % 2 else "f32"
    kind = "generic" if seed % 3 == 0 else "orth"
    blocks = gi.make_blocks(d, radices, kind, rng)
    signs = gi.make_signs(d, rng) if seed % 4 else None
    X = rng.standard_normal((n, d)).astype(np.float32)
    G = rng.standard_normal((n, d)).astype(np.float32)
    if dtype == "bf16":
        X, G = gi.round_to_bf16(X), gi.round_to_bf16(G)
    plan = harp.Plan(d, radices, blocks, signs)
    say(f"random gradients seed={seed} d={d} radices={radices} n={n} {dtype}")
    dK, dX = harp.harp_grad_blocks(plan, to_device(X, dtype), to_device(G, dtype))
    torch.cuda.synchronize()
    rK, rX = ho.grad_blocks(X, G, d, radices, blocks, signs)
    scale = float(np.sqrt((X.astype(np.float64) ** 2).sum(axis=0).max() *
                          (G.astype(np.float64) ** 2).sum(axis=0).max()))
    for t, (a, r) in enumerate(zip(dK, rK)):
        a = a.detach().cpu().numpy().astype(np.float64)
        # float32 sums of n products: 2e-5 of the Cauchy-Schwarz scale plus 1e-5 relative; with
        # generic (non-orthogonal) blocks the activations grow, which the scale of x_t reflects
        tol = 2e-5 * max(scale, float(np.abs(r).max())) + 1e-5 * np.abs(r)
        assert np.all(np.abs(a - r) <= tol), f"stage {t}: {np.abs(a - r).max():.3e}"
    assert_parity(to_host64(dX), rX, dtype, "dX",
                  mag=summand_magnitude(G, d, radices, blocks, transpose=True) if kind == "generic" else None)
    plan.destroy()
