"""harp_apply_noalloc (the entry point for callers that cannot allocate device memory) against
harp_apply / harp_apply_transpose, through the C ABI: same kernels, so the results must be
bit-identical; two calls in a row, the second with a smaller batch, on the library's one array."""
import sys

import numpy as np
import pytest

from paper_2605_29843_amd import inputs as gi
from parity_util import to_device

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def harp():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_29843_amd import harp as h
    return h


def say(*a):
    print("[case]", *a, file=sys.stderr, flush=True)


@pytest.mark.parametrize("d,radices,n1,n2,dtype", [
    (14336, [2] * 11 + [7], 300, 37, "bf16"),       # two launches: pipelined chunks + streamed radix 7
    (11008, [2] * 8 + [43], 500, 64, "bf16"),       # wave kernel + matrix-core stage
    (13824, [2] * 9 + [3, 3, 3], 200, 1, "f32"),    # three launches, the middle one in place
    (4096, [2] * 12, 700, 9, "bf16"),               # one launch: no intermediate at all
])
def test_noalloc_matches_apply_on_two_calls_in_a_row(harp, d, radices, n1, n2, dtype):
    import torch
    rng = np.random.default_rng(d + n1)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng), gi.make_signs(d, rng))
    assert n1 <= harp.harp_apply_noalloc_max_rows(plan)
    for transpose in (False, True):
        ref_fn = harp.harp_apply_transpose if transpose else harp.harp_apply
        for n in (n1, n2):                       # the second call is the smaller one
            X = rng.standard_normal((n, d)).astype(np.float32)
            if dtype == "bf16":
                X = gi.round_to_bf16(X)
            Xd = to_device(X, dtype)
            Y = torch.full_like(Xd, 3.0)
            say(f"noalloc d={d} n={n} {dtype} transpose={transpose} kernel={plan.kernel_name(n)}")
            harp.harp_apply_noalloc(plan, Xd, Y, transpose=transpose)
            ref = ref_fn(plan, Xd)
            torch.cuda.synchronize()
            assert torch.equal(Y, ref), f"n={n} transpose={transpose}: differs from the allocating entry point"
    plan.destroy()


def test_noalloc_refuses_a_batch_beyond_its_array(harp):
    import torch
    d, radices = 14336, [2] * 11 + [7]
    rng = np.random.default_rng(3)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng))
    cap = harp.harp_apply_noalloc_max_rows(plan)
    assert cap == (32 << 20) // (d * 4)
    X = torch.zeros(cap + 1, d, dtype=torch.bfloat16, device="cuda")
    Y = torch.empty_like(X)
    with pytest.raises(harp.HarpError) as e:
        harp.harp_apply_noalloc(plan, X, Y)
    assert e.value.status == harp.HARP_ERR_UNSUPPORTED
    harp.harp_apply_noalloc(plan, X[:cap], Y[:cap])      # exactly the limit is accepted
    torch.cuda.synchronize()
    assert torch.equal(Y[:cap], harp.harp_apply(plan, X[:cap]))
    plan.destroy()
