"""C-ABI boundary on a GPU-less host: the library loads, exports every declared symbol, and
turns every argument error into its status code before touching HIP."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2605_29843_amd", "libharp.so")

if not os.path.exists(LIB):   # built by __graft_entry__.build(); build on demand for local runs
    from paper_2605_29843_amd import build as _b
    _b.build(verbose=False)

from paper_2605_29843_amd import harp  # noqa: E402
from paper_2605_29843_amd import inputs as gi  # noqa: E402

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "harp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(harp_[a-z0-9_]+)\s*\(", text))
    assert {"harp_plan_create", "harp_apply", "harp_apply_transpose", "harp_rotate_weight"} <= declared
    lib = C.CDLL(LIB)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in harp.h but not exported"
    assert declared == set(harp.EXPORTS), declared ^ set(harp.EXPORTS)


def test_status_strings_and_version():
    assert harp.harp_status_string(harp.HARP_OK) == "ok"
    seen = {harp.harp_status_string(s) for s in range(7)}
    assert len(seen) == 7
    assert "gfx950" in harp.harp_version()


def test_greedy_schedule_matches_printed_examples():
    for line in open(os.path.join(GOLD, "greedy_schedule.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        d, v = line.split(":")
        assert harp.harp_greedy_schedule(int(d)) == [int(x) for x in v.split()]
    for line in open(os.path.join(GOLD, "radix_ablation_stage_counts.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        b, cnt = (int(x) for x in line.split(":"))
        assert len(harp.harp_greedy_schedule(4096, b, b)) == cnt
    # other Llama sizes: valid schedules, preferred radix first, leftover prime last
    assert harp.harp_greedy_schedule(11008) == [8, 8, 4, 43]
    assert harp.harp_greedy_schedule(14336) == [8, 8, 8, 7, 4]
    assert harp.harp_greedy_schedule(28672) == [8, 8, 8, 8, 7]
    for d in (2, 3, 97, 5120, 12288, 8192, 13824):
        s = harp.harp_greedy_schedule(d)
        assert int(np.prod(s)) == d and min(s) >= 2
    with pytest.raises(harp.HarpError) as e:
        harp.harp_greedy_schedule(1)
    assert e.value.status == harp.HARP_ERR_INVALID_ARG


def test_greedy_schedule_library_and_oracle_agree_on_many_dimensions():
    """The library derives the schedule from a property (multiplicity of the preferred radix,
    then repeatedly the largest divisor up to b_max), the oracle walks the appendix's procedure:
    two formulations, one answer, over every d up to 3000 and several (b_base, b_max)."""
    from oracle import harp_oracle as ho
    for b_base, b_max in ((8, 8), (2, 2), (4, 8), (16, 16), (8, 4), (3, 7), (8, 64)):
        for d in list(range(2, 3001)) + [11008, 13824, 14336, 28672, 2 ** 20, 3 * 2 ** 19, 97 * 89 * 8]:
            assert harp.harp_greedy_schedule(d, b_base, b_max) == ho.greedy_schedule(d, b_base, b_max), \
                (d, b_base, b_max)


def test_kronecker_plan_argument_errors_come_before_any_device_work():
    lib = harp.lib
    H = gi.hadamard_table(12)
    rad = (C.c_int32 * 8)(*([2] * 8))
    blocks2 = gi.make_blocks(256, [2] * 8, "orth", np.random.default_rng(0))
    bp = (C.c_void_p * 8)(*[b.ctypes.data for b in blocks2])
    out = C.c_void_p(None)

    def call(K, table, n2=256, m2=8, flags=0):
        return lib.harp_plan_create_kronecker(C.byref(out), K, table.ctypes.data if table is not None else None,
                                              n2, m2, rad, bp, None, flags)
    assert call(12, None) == harp.HARP_ERR_INVALID_ARG
    assert call(1, H) == harp.HARP_ERR_INVALID_ARG
    assert call(12, H, flags=harp.HARP_BLOCKS_ON_DEVICE) == harp.HARP_ERR_INVALID_ARG
    assert call(12, H, n2=250) == harp.HARP_ERR_BAD_SCHEDULE
    bad = H.copy()
    bad[3, 4] = 0.5
    assert call(12, bad) == harp.HARP_ERR_INVALID_ARG
    notorth = H.copy()
    notorth[0, :] = 1.0
    notorth[1, :] = 1.0
    assert call(12, notorth) == harp.HARP_ERR_NOT_ORTHOGONAL
    assert call(65, np.ones((65, 65), np.float32)) == harp.HARP_ERR_UNSUPPORTED
    assert out.value is None
    assert lib.harp_plan_tied_slices(None) == -1


def test_hadamard_table_generator():
    for K in (2, 4, 12, 20, 28, 36, 64):
        H = gi.hadamard_table(K).astype(np.float64)
        assert set(np.unique(H)) <= {-1.0, 1.0}
        np.testing.assert_array_equal(H @ H.T, K * np.eye(K))
    with pytest.raises(ValueError):
        gi.hadamard_table(6)


def test_make_blocks_kinds():
    """'generic' blocks are really non-orthogonal (and well conditioned); unknown kinds raise."""
    rng = np.random.default_rng(0)
    for b in (2, 3, 8, 43):
        K = gi.make_blocks(b * 16, [b], "generic", rng)[0].astype(np.float64)
        dev = np.abs(np.swapaxes(K, 1, 2) @ K - np.eye(b)).max(axis=(1, 2))
        assert dev.min() > 0.02
        sv = np.linalg.svd(K, compute_uv=False)
        assert sv.min() > 0.1 and sv.max() < 3.0
        Q = gi.make_blocks(b * 16, [b], "orth", rng)[0].astype(np.float64)
        assert np.abs(np.swapaxes(Q, 1, 2) @ Q - np.eye(b)).max() < 1e-6
    with pytest.raises(ValueError):
        gi.make_blocks(16, [4, 4], "general", rng)


def _status_of_create(d, radices, blocks, signs=None, flags=0):
    try:
        p = harp.Plan(d, radices, blocks, signs, flags)
    except harp.HarpError as e:
        return e.status
    p.destroy()
    return harp.HARP_OK


def test_plan_create_rejects_bad_schedules_before_any_device_work():
    rng = np.random.default_rng(0)
    good = gi.make_blocks(16, [4, 4], "orth", rng)
    assert _status_of_create(16, [4, 2], good) == harp.HARP_ERR_BAD_SCHEDULE      # product != d
    assert _status_of_create(16, [16, 1], good) == harp.HARP_ERR_BAD_SCHEDULE     # radix < 2
    assert _status_of_create(16, [], []) == harp.HARP_ERR_BAD_SCHEDULE            # no stage
    assert _status_of_create(1, [1], good[:1]) == harp.HARP_ERR_INVALID_ARG       # d < 2
    assert _status_of_create(16, [4, 4], [good[0], None]) == harp.HARP_ERR_INVALID_ARG
    assert _status_of_create(16, [4, 4], good, flags=64) == harp.HARP_ERR_INVALID_ARG
    bad_signs = np.array([1] * 15 + [0], dtype=np.int8)
    assert _status_of_create(16, [4, 4], good, bad_signs) == harp.HARP_ERR_INVALID_ARG
    nan_blocks = [good[0].copy(), good[1].copy()]
    nan_blocks[1][2, 1, 1] = np.nan
    assert _status_of_create(16, [4, 4], nan_blocks) == harp.HARP_ERR_INVALID_ARG
    big = gi.make_blocks(2 * 67, [2, 67], "orth", rng)
    assert _status_of_create(134, [2, 67], big) == harp.HARP_ERR_UNSUPPORTED      # radix > 64
    # non-orthogonal block: accepted without the flag, rejected with it
    skew = [good[0].copy(), good[1].copy()]
    skew[0][1] *= 1.01
    assert _status_of_create(16, [4, 4], skew, flags=harp.HARP_VALIDATE_ORTHO) == \
        harp.HARP_ERR_NOT_ORTHOGONAL
    ok = _status_of_create(16, [4, 4], good, flags=harp.HARP_VALIDATE_ORTHO)
    assert ok == (harp.HARP_OK if _have_gpu() else harp.HARP_ERR_DEVICE)


def test_null_plan_and_null_out_are_invalid_arguments():
    lib = harp.lib
    assert lib.harp_apply(None, None, 4, None, 4, 1, harp.HARP_F32, None) == harp.HARP_ERR_INVALID_ARG
    assert lib.harp_apply_transpose(None, None, 4, None, 4, 1, 0, None) == harp.HARP_ERR_INVALID_ARG
    assert lib.harp_plan_destroy(None) == harp.HARP_OK
    assert lib.harp_plan_dim(None) == -1
    assert lib.harp_plan_num_stages(None) == -1
    assert lib.harp_plan_param_count(None) == -1
    assert lib.harp_plan_set_algo(None, 0) == harp.HARP_ERR_INVALID_ARG
    rad = (C.c_int32 * 1)(2)
    ptr = (C.c_void_p * 1)(None)
    assert lib.harp_plan_create(None, 2, 1, rad, ptr, None, 0) == harp.HARP_ERR_INVALID_ARG
    b = C.c_size_t(123)
    assert lib.harp_rotate_weight_workspace_size(None, None, 8, 8, 7, C.byref(b)) == \
        harp.HARP_ERR_INVALID_ARG
    assert lib.harp_rotate_weight_workspace_size(None, None, 8, 8, harp.HARP_BF16, C.byref(b)) == \
        harp.HARP_OK and b.value == 0
    # identity on both sides with nothing to copy is a no-op
    assert lib.harp_rotate_weight(None, None, None, 0, None, 0, 0, 0, harp.HARP_F32, None, 0,
                                  None) == harp.HARP_OK
    assert lib.harp_rotate_weight(None, None, None, 8, None, 8, 8, 8, harp.HARP_F32, None, 0,
                                  None) == harp.HARP_ERR_INVALID_ARG


def test_grad_blocks_argument_errors_without_a_gpu():
    lib = harp.lib
    b = C.c_size_t(5)
    assert lib.harp_grad_blocks_workspace_size(None, 4, C.byref(b)) == harp.HARP_ERR_INVALID_ARG
    assert lib.harp_grad_blocks(None, None, 0, None, 0, 0, harp.HARP_F32, None, None, 0, None, 0,
                                None) == harp.HARP_ERR_INVALID_ARG


def test_blocks_from_theta_host_front_end_matches_the_oracle():
    """The library's parameter front end runs on the host, so it is checked here without a GPU:
    Givens (radix 2) and Cayley (radix > 2) blocks, Hadamard / identity / custom mixers."""
    import numpy as np
    from oracle import harp_oracle as ho
    rng = np.random.default_rng(11)
    d, radices = 480, [2, 8, 3, 2, 5]
    G3 = np.linalg.qr(rng.standard_normal((3, 3)))[0].astype(np.float32)
    thetas = [(1.5 * rng.standard_normal((d // b, b * (b - 1) // 2))).astype(np.float32) for b in radices]
    thetas[3] = None
    mixers = [None, "hadamard", G3, "identity", "identity"]
    got = harp.harp_blocks_from_theta(d, radices, thetas, mixers)
    ref = ho.blocks_from_theta(d, radices, thetas, mixers)
    for g, r in zip(got, ref):
        assert g.dtype == np.float32 and g.shape == r.shape
        assert np.max(np.abs(g - r)) <= 2.0 ** -23          # one float32 rounding of an entry <= 1
    # Theta = 0: exactly the normalised Hadamard block
    H = harp.harp_blocks_from_theta(64, [8, 8])
    np.testing.assert_array_equal(H[0][5], ho.sylvester_hadamard(8).astype(np.float32))
    # argument errors
    with pytest.raises(harp.HarpError) as e:
        harp.harp_blocks_from_theta(6, [2, 3])              # Hadamard mixer at radix 3
    assert e.value.status == harp.HARP_ERR_INVALID_ARG
    bad = [np.full((3, 1), np.nan, np.float32), None]
    with pytest.raises(harp.HarpError) as e:
        harp.harp_blocks_from_theta(6, [2, 3], bad, [None, "identity"])
    assert e.value.status == harp.HARP_ERR_INVALID_ARG
    with pytest.raises(harp.HarpError) as e:
        harp.harp_blocks_from_theta(10, [2, 3])
    assert e.value.status == harp.HARP_ERR_BAD_SCHEDULE


def test_theta_int8_host_front_end_matches_the_oracle_bit_for_bit():
    """Codes and scales are decided in float32 on both sides, so they must agree exactly."""
    import numpy as np
    from oracle import harp_oracle as ho
    rng = np.random.default_rng(23)
    d, radices = 1680, [2, 8, 3, 5, 7]
    thetas = [(rng.standard_normal((d // b, b * (b - 1) // 2)) * rng.uniform(1e-4, 4.0, (d // b, 1)))
              .astype(np.float32) for b in radices]
    thetas[2][7] = 0.0                                     # an all-zero block: scale 0, codes 0
    thetas[0][3, 0] = np.float32(63.5 / 127.0)             # neighbours of rounding ties
    codes, scales = harp.harp_theta_quantize_int8(d, radices, thetas)
    rc, rs = ho.quantize_theta_int8(d, radices, thetas)
    for t in range(len(radices)):
        np.testing.assert_array_equal(codes[t], rc[t])
        np.testing.assert_array_equal(scales[t], rs[t])
    assert scales[2][7] == 0.0 and not codes[2][7].any()
    back = harp.harp_theta_dequantize_int8(d, radices, codes, scales)
    rb = ho.dequantize_theta_int8(d, radices, rc, rs)
    for t in range(len(radices)):
        np.testing.assert_array_equal(back[t], rb[t])
    # argument errors: a code outside the quantiser's range, a negative scale, a NaN parameter
    bad = [c.copy() for c in codes]
    bad[1][0, 0] = -128
    with pytest.raises(harp.HarpError) as e:
        harp.harp_theta_dequantize_int8(d, radices, bad, scales)
    assert e.value.status == harp.HARP_ERR_INVALID_ARG
    bads = [x.copy() for x in scales]
    bads[0][0] = -1.0
    with pytest.raises(harp.HarpError) as e:
        harp.harp_theta_dequantize_int8(d, radices, codes, bads)
    assert e.value.status == harp.HARP_ERR_INVALID_ARG
    nan = [x.copy() for x in thetas]
    nan[4][0, 0] = np.nan
    with pytest.raises(harp.HarpError) as e:
        harp.harp_theta_quantize_int8(d, radices, nan)
    assert e.value.status == harp.HARP_ERR_INVALID_ARG
    with pytest.raises(harp.HarpError) as e:
        harp.harp_theta_quantize_int8(10, [2, 3], [np.zeros((5, 1), np.float32), np.zeros((3, 3), np.float32)])
    assert e.value.status == harp.HARP_ERR_BAD_SCHEDULE


def test_kronecker_blocks_expand_to_the_kronecker_product():
    """Host expansion of the Kronecker fallback, checked through the oracle's explicit dense
    construction: U_d == kron(table / sqrt(K), U_{n2})."""
    import numpy as np
    from oracle import harp_oracle as ho
    rng = np.random.default_rng(5)
    n2, radices2 = 16, [2, 4, 2]
    blocks2 = gi.make_blocks(n2, radices2, "orth", rng)
    # a 12 x 12 Hadamard-like table (Paley construction, q = 11) and the 2 x 2 one
    q = 11
    res = {(x * x) % q for x in range(1, q)}
    Q = np.array([[0 if i == j else (1 if ((i - j) % q) in res else -1) for j in range(q)] for i in range(q)])
    S = np.zeros((q + 1, q + 1), dtype=np.int64)
    S[0, 1:] = 1
    S[1:, 0] = -1
    S[1:, 1:] = Q
    H12 = (np.eye(q + 1, dtype=np.int64) + S).astype(np.float32)
    assert np.array_equal(H12 @ H12.T, 12 * np.eye(12))
    for table in (np.array([[1, 1], [1, -1]], np.float32), H12):
        K = table.shape[0]
        radices, blocks = harp.harp_kronecker_blocks(table, n2, radices2, blocks2)
        assert radices == radices2 + [K]
        U = ho.U_explicit(K * n2, radices, blocks)
        U2 = ho.U_explicit(n2, radices2, blocks2)
        np.testing.assert_allclose(U, np.kron(table.astype(np.float64) / np.sqrt(K), U2), atol=1e-6)
    bad = np.array([[1, 1], [1, 1]], np.float32)
    with pytest.raises(harp.HarpError) as e:
        harp.harp_kronecker_blocks(bad, n2, radices2, blocks2)
    assert e.value.status == harp.HARP_ERR_NOT_ORTHOGONAL
    with pytest.raises(harp.HarpError) as e:
        harp.harp_kronecker_blocks(np.array([[1, 0.5], [1, -1]], np.float32), n2, radices2, blocks2)
    assert e.value.status == harp.HARP_ERR_INVALID_ARG

