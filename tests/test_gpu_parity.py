"""GPU parity: libharp (through its C ABI) against the float64 CPU oracle, element by element,
on the same seeded inputs.  Every test prints the case it is about to launch."""
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
    assert torch.cuda.is_available(), "GPU tests need a device"
    from paper_2605_29843_amd import harp as h     # raises if libharp.so is missing
    return h


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


def run_case(harp, d, radices, n, dtype, kind="orth", seed=0, algo=None, ld_pad=0, rows=None,
             with_signs=True, act=None, both=True):
    import torch
    rng = np.random.default_rng(seed)
    blocks = gi.make_blocks(d, radices, kind, rng)
    signs = gi.make_signs(d, rng) if with_signs else None
    X = rng.standard_normal((n, d)).astype(np.float32) if act is None else act
    if dtype == "bf16":
        X = gi.round_to_bf16(X)
    plan = harp.Plan(d, radices, blocks, signs)
    if algo is not None:
        plan.set_algo(algo)
    if rows is not None:
        plan.set_rows_per_tile(rows)
    say(f"d={d} radices={radices} n={n} {dtype} kind={kind} algo={algo} ld_pad={ld_pad} rows={rows} "
        f"kernel={plan.kernel_name()}")
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Xd_full = torch.zeros((n, d + ld_pad), dtype=tdt, device="cuda")
    Xd = Xd_full[:, :d]
    Xd.copy_(to_device(X, dtype))
    Yd_full = torch.full((n, d + ld_pad), 7.0, dtype=tdt, device="cuda")
    Yd = Yd_full[:, :d]
    out = {}
    harp.harp_apply(plan, Xd, Yd)
    torch.cuda.synchronize()
    Y = to_host64(Yd)
    generic = (kind == "generic")    # non-orthogonal blocks: rounding is relative to the summands
    if n > 0:
        Yref = ho.apply_staged(X, d, radices, blocks, signs)
        out["apply"] = assert_parity(Y, Yref, dtype, "apply",
                                     mag=summand_magnitude(X, d, radices, blocks) if generic else None)
    if ld_pad:
        assert torch.all(Yd_full[:, d:] == 7.0), "padding columns were written"
    if both:
        Zd_full = torch.full((n, d + ld_pad), 7.0, dtype=tdt, device="cuda")
        Zd = Zd_full[:, :d]
        harp.harp_apply_transpose(plan, Xd, Zd)
        torch.cuda.synchronize()
        if n > 0:
            Zref = ho.apply_transpose_staged(X, d, radices, blocks, signs)
            out["transpose"] = assert_parity(
                to_host64(Zd), Zref, dtype, "apply_transpose",
                mag=summand_magnitude(X, d, radices, blocks, transpose=True) if generic else None)
    plan.destroy()
    return out


# ------------------------------------------------------------------ config 1: tiny
@pytest.mark.parametrize("algo", [1, 2])
@pytest.mark.parametrize("kind", ["orth", "hadamard"])
def test_tiny_256_radix2_fp32(harp, algo, kind):
    w = gi.workload("tiny_256_r2", kind=kind)
    import torch
    plan = harp.Plan(w["d"], w["radices"], w["blocks"], w["signs"])
    plan.set_algo(algo)
    say("tiny_256_r2", kind, "algo", algo)
    Xd = to_device(w["X"], "f32")
    U = ho.build_U(w["d"], w["radices"], w["blocks"], w["signs"])     # the dense definition
    Y = to_host64(harp.harp_apply(plan, Xd))
    assert_parity(Y, w["X"].astype(np.float64) @ U, "f32", "apply")
    Z = to_host64(harp.harp_apply_transpose(plan, Xd))
    assert_parity(Z, w["X"].astype(np.float64) @ U.T, "f32", "transpose")
    # round trip on the device
    back = to_host64(harp.harp_apply_transpose(plan, harp.harp_apply(plan, Xd)))
    assert np.max(np.abs(back - w["X"])) < 1e-5 * np.max(np.abs(w["X"])) * 4
    torch.cuda.synchronize()
    plan.destroy()


# ------------------------------------------------------------------ every pass kind, ragged tiles
SMALL_CASES = [
    ([2] * 5 + [3], 13), ([4, 4, 4], 9), ([8, 8], 17), ([3, 5, 7], 11), ([2, 2, 7, 2], 5),
    ([16, 4], 33), ([43, 2, 2], 7), ([2] * 8 + [43], 19), ([5, 2, 3], 1), ([2], 3), ([64], 4),
    ([2] * 11, 10), ([6, 9, 11], 6), ([2, 2, 2, 2, 2, 2, 2], 70),
]


@pytest.mark.parametrize("radices,n", SMALL_CASES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("algo", [1, 2])
def test_small_schedules_all_kinds(harp, radices, n, dtype, algo):
    d = int(np.prod(radices))
    run_case(harp, d, radices, n, dtype, kind="orth", seed=d + n, algo=algo)


@pytest.mark.parametrize("kind", ["qr", "hadamard"])
def test_dense_2x2_blocks_and_reflections(harp, kind):
    """'qr' radix-2 blocks include reflections -> the 4-value 2x2 path; non-orthogonal too."""
    run_case(harp, 512, [2] * 9, 21, "f32", kind=kind, seed=5, algo=2)
    run_case(harp, 96, [2, 2, 2, 2, 2, 3], 9, "bf16", kind=kind if kind == "qr" else "orth", seed=6, algo=2)


def test_non_orthogonal_blocks_are_still_the_linear_map(harp):
    import torch
    d, radices, n = 120, [2, 3, 4, 5], 6
    rng = np.random.default_rng(8)
    blocks = [rng.standard_normal((d // b, b, b)).astype(np.float32) for b in radices]
    signs = gi.make_signs(d, rng)
    X = rng.standard_normal((n, d)).astype(np.float32)
    for algo in (1, 2):
        plan = harp.Plan(d, radices, blocks, signs)
        plan.set_algo(algo)
        say("non-orthogonal", radices, "algo", algo)
        U = ho.U_explicit(d, radices, blocks, signs)
        Y = to_host64(harp.harp_apply(plan, to_device(X, "f32")))
        Z = to_host64(harp.harp_apply_transpose(plan, to_device(X, "f32")))
        torch.cuda.synchronize()
        scale = np.abs(X.astype(np.float64)) @ np.abs(U)        # magnitude of the summands
        assert np.max(np.abs(Y - X @ U) / scale) < 2e-6
        assert np.max(np.abs(Z - X @ U.T) / (np.abs(X.astype(np.float64)) @ np.abs(U.T))) < 2e-6
        plan.destroy()


def _radix2_plan_with_special_blocks(d, m, special, seed):
    """Random Givens blocks; in every stage every 7th block is replaced by `special(c)`."""
    rng = np.random.default_rng(seed)
    radices = [2] * m
    blocks = gi.make_blocks(d, radices, "orth", rng)
    for t in range(m):
        for c in range(t % 7, d // 2, 7):
            blocks[t][c] = special(c)
    return radices, blocks, gi.make_signs(d, rng)


@pytest.mark.parametrize("d", [256, 4096])
@pytest.mark.parametrize("case", ["quarter_turn", "swap", "near_quarter_turn", "tiny_diagonal", "general",
                                  "diagonal_1e-6", "diagonal_1e-9", "diagonal_1e-11"])
def test_radix2_blocks_with_zero_or_tiny_diagonal(harp, d, case):
    """The two-shear form divides by the diagonal of a block: blocks with an exactly zero
    diagonal (quarter turns, swaps) must take the lifting fallback, nearly zero ones and
    general invertible 2x2 blocks must stay accurate."""
    import torch
    m = int(np.log2(d))
    eps = 3e-5
    special = {
        "quarter_turn": lambda c: np.array([[0, -1], [1, 0]] if c % 2 else [[0, 1], [-1, 0]], np.float32),
        "swap": lambda c: np.array([[0, 1], [1, 0]], np.float32),
        "near_quarter_turn": lambda c: np.array([[np.sin(eps), -np.cos(eps)], [np.cos(eps), np.sin(eps)]],
                                                np.float32),
        # diagonal 1e-13: the shear factor would be 1e13, beyond the plan builder's bound
        "tiny_diagonal": lambda c: np.array([[1e-13, -1.0], [1.0, 1e-13]], np.float32),
        "general": lambda c: np.array([[1.5, 0.25 * (c % 5)], [-0.5, 0.75]], np.float32),
        # the range in between: the two-shear form is still taken, with shear factors of
        # 1e6 .. 1e11 and pending scales that accumulate over the stages (or the builder falls
        # back when a scale leaves its range): either way the result must stay accurate
        "diagonal_1e-6": lambda c: np.array([[1e-6, -1.0], [1.0, 1e-6]], np.float32),
        "diagonal_1e-9": lambda c: np.array([[1e-9, 1.0], [-1.0, 1e-9]] if c % 2 else
                                            [[1e-9, -1.0], [1.0, 1e-9]], np.float32),
        "diagonal_1e-11": lambda c: np.array([[1e-11, -1.0], [1.0, -1e-11 if c % 3 == 0 else 1e-11]],
                                             np.float32),
    }[case]
    radices, blocks, signs = _radix2_plan_with_special_blocks(d, m, special, seed=d + len(case))
    n = 37
    X = gi.round_to_bf16(np.random.default_rng(3).standard_normal((n, d)).astype(np.float32))
    for dtype in ("bf16", "f32"):
        plan = harp.Plan(d, radices, blocks, signs)
        say(f"special blocks {case} d={d} {dtype} kernel={plan.kernel_name()}")
        Xd = to_device(X, dtype)
        Y = to_host64(harp.harp_apply(plan, Xd))
        Z = to_host64(harp.harp_apply_transpose(plan, Xd))
        torch.cuda.synchronize()
        Yref = ho.apply_staged(X, d, radices, blocks, signs)
        Zref = ho.apply_transpose_staged(X, d, radices, blocks, signs)
        if case == "general":      # not orthogonal: error relative to the output's row scale
            for got, ref in ((Y, Yref), (Z, Zref)):
                rho = np.linalg.norm(ref, axis=1, keepdims=True) / np.sqrt(d)
                tol = 1e-5 if dtype == "f32" else 8e-3
                assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rho)) < tol
        else:
            assert_parity(Y, Yref, dtype, "apply")
            assert_parity(Z, Zref, dtype, "apply_transpose")
        plan.destroy()


# ------------------------------------------------------------------ layout edge cases
def test_empty_batch_is_a_noop(harp):
    run_case(harp, 64, [2] * 6, 0, "bf16", algo=2)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_leading_dimension_padding_and_unaligned_rows(harp, dtype):
    run_case(harp, 256, [2] * 8, 19, dtype, ld_pad=24, seed=3)      # aligned padding
    run_case(harp, 256, [2] * 8, 19, dtype, ld_pad=3, seed=4)       # rows not 16-byte aligned
    run_case(harp, 105, [3, 5, 7], 8, dtype, ld_pad=1, seed=5)      # odd d: scalar I/O path


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_in_place(harp, dtype):
    import torch
    d, radices, n = 1024, [2] * 10, 37
    rng = np.random.default_rng(12)
    blocks = gi.make_blocks(d, radices, "orth", rng)
    signs = gi.make_signs(d, rng)
    X = rng.standard_normal((n, d)).astype(np.float32)
    if dtype == "bf16":
        X = gi.round_to_bf16(X)
    plan = harp.Plan(d, radices, blocks, signs)
    say("in place", d, n, dtype)
    Xd = to_device(X, dtype)
    harp.harp_apply(plan, Xd, Xd)
    torch.cuda.synchronize()
    assert_parity(to_host64(Xd), ho.apply_staged(X, d, radices, blocks, signs), dtype, "in place")
    plan.destroy()


@pytest.mark.parametrize("rows", [1, 2, 3, 5, 8])
def test_rows_per_tile_override_with_ragged_tail(harp, rows):
    run_case(harp, 2048, [2] * 11, 29, "bf16", seed=rows, rows=rows)


# ------------------------------------------------------------------ config 2: d = 4096
@pytest.mark.parametrize("radices", [[2] * 12, [8] * 4, [4] * 6, [16] * 3], ids=["r2", "r8", "r4", "r16"])
def test_llama7b_hidden_4096_dense_oracle(harp, radices):
    """n = 96 rows (several tiles + ragged tail) against the dense definition X @ U."""
    import torch
    d, n = 4096, 91
    blocks, signs = gi.processor(d, radices, config=2)
    X = gi.activations(n, d, config=2)
    plan = harp.Plan(d, radices, blocks, signs)
    say("4096 dense oracle", radices, plan.kernel_name())
    U = ho.build_U(d, radices, blocks, signs)
    Xd = to_device(X, "bf16")
    Y = to_host64(harp.harp_apply(plan, Xd))
    Z = to_host64(harp.harp_apply_transpose(plan, Xd))
    torch.cuda.synchronize()
    assert_parity(Y, X.astype(np.float64) @ U, "bf16", "apply")
    assert_parity(Z, X.astype(np.float64) @ U.T, "bf16", "transpose")
    plan.destroy()


@pytest.mark.parametrize("n,rows", [(1, None), (2, None), (3, 2), (5, 1), (37, 7), (91, None), (300, 32),
                                    (64, 64)])
@pytest.mark.parametrize("with_signs", [True, False])
def test_pipelined_radix2_kernel_4096(harp, n, rows, with_signs):
    """d = 4096, twelve rotation stages, bf16: the row-pipelined kernel at ragged tile sizes
    (fill/drain of the three-stage pipeline with fewer rows than pipeline stages, too)."""
    X = gi.activations(n, 4096, config=2)
    out = run_case(harp, 4096, [2] * 12, n, "bf16", seed=100 + n, rows=rows, with_signs=with_signs,
                   act=X)
    assert set(out) == {"apply", "transpose"}


@pytest.mark.parametrize("d,dtype,n", [(2048, "bf16", 45), (2048, "f32", 19), (4096, "f32", 33),
                                       (2048, "bf16", 1), (4096, "f32", 2), (2048, "bf16", 1031),
                                       (2048, "bf16", 2)])
def test_pipelined_kernel_other_sizes_and_types(harp, d, dtype, n):
    radices = [2] * int(np.log2(d))
    rng = np.random.default_rng(d + n)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng))
    # bf16 rows: two wave groups with in-wave (DPP) digit exchanges; float32 rows: three groups
    assert plan.kernel_name(n, harp.HARP_BF16) == "dpp_radix2"
    assert plan.kernel_name(n, harp.HARP_F32) == "pipe_radix2"
    plan.destroy()
    run_case(harp, d, radices, n, dtype, seed=d + n)


@pytest.mark.parametrize("d,n", [(256, 70), (512, 33), (1024, 129), (256, 1), (1024, 3), (1024, 2500)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_wave_local_kernel_short_rows(harp, d, n, dtype):
    """Radix-2 chains on rows of 256 / 512 / 1024: one wave per 1024-coordinate window."""
    radices = [2] * int(np.log2(d))
    rng = np.random.default_rng(d)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng))
    # (bf16 rows of 1024: the two-group DPP kernel, one wave per group)
    assert plan.kernel_name(n, harp.HARP_F32) == "wave_radix2"
    assert plan.kernel_name(n, harp.HARP_BF16) == ("dpp_radix2" if d == 1024 else "wave_radix2")
    plan.destroy()
    run_case(harp, d, radices, n, dtype, seed=d + n)
    run_case(harp, d, radices, n, dtype, seed=d + n + 1, rows=3, with_signs=False)


def test_pipelined_kernel_is_selected_and_in_place(harp):
    import torch
    d, radices, n = 4096, [2] * 12, 77
    blocks, signs = gi.processor(d, radices, config=2)
    X = gi.activations(n, d, config=2)
    plan = harp.Plan(d, radices, blocks, signs)
    assert plan.kernel_name() == "dpp_radix2"
    say("pipe in place", n)
    Xd = to_device(X, "bf16")
    harp.harp_apply(plan, Xd, Xd)
    torch.cuda.synchronize()
    assert_parity(to_host64(Xd), ho.apply_staged(X, d, radices, blocks, signs), "bf16", "in place")
    # forcing the generic family takes the other kernel and still matches
    plan.set_algo(1)
    assert plan.kernel_name() == "tile_generic"
    Y = harp.harp_apply(plan, to_device(X, "bf16"))
    torch.cuda.synchronize()
    assert_parity(to_host64(Y), ho.apply_staged(X, d, radices, blocks, signs), "bf16", "generic")
    plan.destroy()


def _full_size(harp, name, row_step=1, dense=False, transpose=True):
    """Full-size workload in the launch configuration the benchmark uses.  Every row (or, with
    row_step = k > 1, one row out of every k consecutive ones at a varying offset, so that every
    row tile of every launch contributes) is compared with the oracle element by element: with
    dense = True against the definition X @ U with U materialised, otherwise against the
    stage-by-stage form.  Norm preservation is checked on every row."""
    import torch
    w = gi.workload(name)
    d, n, radices = w["d"], w["n"], w["radices"]
    plan = harp.Plan(d, radices, w["blocks"], w["signs"])
    say("full size", name, f"n={n} d={d} row_step={row_step} dense={dense}", plan.kernel_name())
    Xd = to_device(w["X"], "bf16")
    Yd = harp.harp_apply(plan, Xd)
    torch.cuda.synchronize()
    if row_step == 1:
        rows = np.arange(n)
    else:
        k = np.arange((n + row_step - 1) // row_step)
        rows = np.minimum(k * row_step + (k * 7 + 3) % row_step, n - 1)
        rows = np.unique(np.concatenate([rows, [0, n - 1]]))
    Xs = w["X"][rows]
    U = ho.build_U(d, radices, w["blocks"], w["signs"]) if dense else None
    idx = torch.from_numpy(rows).cuda()
    Yref = Xs.astype(np.float64) @ U if dense else ho.apply_staged(Xs, d, radices, w["blocks"], w["signs"])
    assert_parity(to_host64(Yd[idx]), Yref, "bf16", name + " apply")
    # property that holds at any size: every row keeps its norm (orthogonal U), up to bf16 rounding
    nx = torch.linalg.vector_norm(Xd.float(), dim=1)
    ny = torch.linalg.vector_norm(Yd.float(), dim=1)
    assert float(torch.max(torch.abs(ny - nx) / nx)) < 2e-3
    if transpose:
        say("full size", name, "transpose")
        Zd = harp.harp_apply_transpose(plan, Xd)
        torch.cuda.synchronize()
        Zref = Xs.astype(np.float64) @ U.T if dense else \
            ho.apply_transpose_staged(Xs, d, radices, w["blocks"], w["signs"])
        assert_parity(to_host64(Zd[idx]), Zref, "bf16", name + " transpose")
        nz = torch.linalg.vector_norm(Zd.float(), dim=1)
        assert float(torch.max(torch.abs(nz - nx) / nx)) < 2e-3
    plan.destroy()


def test_full_size_4096_every_row_against_dense_U(harp):
    """The benchmark's batch (2048 x 4096 bf16, twelve radix-2 stages) in the benchmark's launch
    configuration: all 2048 rows of apply and apply_transpose against X @ U and X @ U^T."""
    _full_size(harp, "llama7b_4096_r2", dense=True)


def test_full_size_4096_radix8_every_row(harp):
    _full_size(harp, "llama7b_4096_r8")


# ------------------------------------------------------------------ config 3: mixed radix
@pytest.mark.parametrize("name", ["down_11008_r2x8_43", "ffn_14336_r2x11_7", "llama13b_5120_r2x10_5",
                                  "ffn13b_13824_r2x9_27"])
def test_full_size_mixed_radix(harp, name):
    """All 2048 rows, both directions, against the stage-by-stage oracle."""
    _full_size(harp, name)


@pytest.mark.parametrize("d,radices", [(11008, [8, 8, 4, 43]), (14336, [8, 8, 8, 7, 4]),
                                       (5120, [8, 8, 8, 5, 2]), (12288, [2] * 12 + [3])])
def test_paper_greedy_schedules(harp, d, radices):
    run_case(harp, d, radices, 21, "bf16", seed=d, act=gi.activations(21, d, config=3))


# ------------------------------------------------------------------ split programs (d > 4096)
SPLIT_CASES = [
    (8192, [2] * 13, 70), (5120, [8, 8, 8, 5, 2], 33), (11008, [2] * 8 + [43], 40),
    (11008, [8, 8, 4, 43], 9), (12288, [2] * 12 + [3], 65), (14336, [2] * 11 + [7], 130),
    (28672, [2] * 12 + [7], 37), (16384, [4] * 7, 12), (24576, [2] * 13 + [3], 5),
    (65536, [2] * 16, 6), (3 * 4096 * 5, [2] * 12 + [3, 5], 4),
    # chunk ends behind the radix-2 stages (512); streamed radix-3 stages, two per trip
    (13824, [2] * 9 + [3, 3, 3], 21), (13824, [8, 8, 8, 3, 3, 3], 10), (4608, [2] * 9 + [3, 3], 33),
    (41472, [2] * 9 + [3, 3, 3, 3], 3),
]


@pytest.mark.parametrize("d,radices,n", SPLIT_CASES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_split_program_chunk_plus_stream(harp, d, radices, n, dtype):
    """Low digits fused on chip per chunk, digits above streamed through a float32
    intermediate; also the only path for rows that do not fit in LDS (d = 65536)."""
    X = gi.activations(n, d, config=3, bf16=(dtype == "bf16"))
    run_case(harp, d, radices, n, dtype, seed=d + n, algo=3, act=X)


@pytest.mark.parametrize("d,radices,n", [(12288, [2] * 12 + [3], 3), (14336, [2] * 11 + [7], 2),
                                         (11008, [2] * 8 + [43], 5)])
def test_whole_row_tile_kernel_for_long_rows(harp, d, radices, n):
    """The one-launch whole-row path (algo = fused) stays available for rows longer than a chunk."""
    run_case(harp, d, radices, n, "bf16", seed=d + n, algo=2)


MFMA_CASES = [
    (11008, [2] * 8 + [43], 300), (22528, [2] * 11 + [11], 40), (4096 * 33, [2] * 12 + [33], 5),
    (65536, [4] * 5 + [64], 18), (8192 * 2, [8, 8, 8, 2, 16], 33), (11008, [8, 8, 4, 43], 17),
]


@pytest.mark.parametrize("d,radices,n", MFMA_CASES)
def test_large_radix_stage_on_matrix_cores(harp, d, radices, n):
    """bf16 I/O: the streamed radix >= 9 stage runs on MFMA with bf16-split operands (apply:
    float32 in, bf16 out; transpose: bf16 in, float32 out); ragged row counts."""
    X = gi.activations(n, d, config=3)
    out = run_case(harp, d, radices, n, "bf16", seed=d + n, algo=3, act=X)
    assert max(out.values()) < 0.8      # error stays well inside the bf16 tolerance


@pytest.mark.parametrize("d,radices,n", MFMA_CASES)
def test_large_radix_stage_on_matrix_cores_float32(harp, d, radices, n):
    """float32 I/O: the same stage runs on the float32 MFMA instruction with unsplit
    operands and has to meet the float32 tolerance."""
    X = gi.activations(n, d, config=3, bf16=False)
    run_case(harp, d, radices, n, "f32", seed=d + n + 1, algo=3, act=X)


@pytest.mark.parametrize("d,radices,n", [
    (2816, [8, 8, 4, 11], 37), (1408, [8, 8, 2, 11], 20), (2752, [8, 8, 43], 33),
    (4096, [8, 8, 64], 18), (8192, [8, 8, 16, 8], 9), (4096, [2] * 8 + [16], 70),
    (2304, [4, 4, 4, 4, 9], 5)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_large_radix_stage_ends_the_chunk(harp, d, radices, n, dtype):
    """Rows of at most one chunk whose schedule ends in a leftover prime (or any radix >= 9)
    behind small stages: the default program streams that stage on the matrix cores instead of
    running it on chip; the one-launch program stays selectable and agrees."""
    rng = np.random.default_rng(d)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng))
    assert plan.kernel_name(n).startswith("split"), plan.kernel_name(n)
    plan.destroy()
    X = gi.activations(n, d, config=3, bf16=(dtype == "bf16"))
    run_case(harp, d, radices, n, dtype, seed=d + n, act=X)
    run_case(harp, d, radices, n, dtype, seed=d + n, algo=2, act=X)


@pytest.mark.parametrize("d,k", [(768, 8), (1536, 9), (3072, 10)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_radix2_chain_with_a_radix3_tail_up_to_4096(harp, d, k, dtype):
    """[2]*k + [3] in one chunk: large forward batches take the split program (wave kernel on the
    radix-2 chunk + streamed radix-3 stage), small ones and the transposed direction the
    one-launch kernel; both agree with the oracle."""
    radices = [2] * k + [3]
    rng = np.random.default_rng(d)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng))
    assert plan.kernel_name(2048).startswith("split"), plan.kernel_name(2048)
    assert not plan.kernel_name(64).startswith("split"), plan.kernel_name(64)
    plan.destroy()
    run_case(harp, d, radices, 600, dtype, seed=d + 1, act=gi.activations(600, d, config=3, bf16=(dtype == "bf16")))
    run_case(harp, d, radices, 37, dtype, seed=d + 2, act=gi.activations(37, d, config=3, bf16=(dtype == "bf16")))


def test_chunk_of_a_llama13b_ffn_row_ends_behind_its_radix2_stages(harp):
    """13824 = 2^9 * 27: the default program is the wave kernel on 512-coordinate chunks plus
    streamed radix-3 stages (two of them in one trip), not the general tile kernel on 1536."""
    d, radices = 13824, [2] * 9 + [3, 3, 3]
    rng = np.random.default_rng(7)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng))
    assert plan.kernel_name(2048, harp.HARP_F32) == "split_wave_stream", plan.kernel_name(2048, harp.HARP_F32)
    # (bf16 callers: the same kernels with the half-precision intermediate on both trips)
    assert plan.kernel_name(2048, harp.HARP_BF16) == "split_wave_stream_h16"
    plan.destroy()
    run_case(harp, d, radices, 19, "f32", seed=77, act=gi.activations(19, d, config=3, bf16=False))


@pytest.mark.parametrize("d,radices", [
    (12288, [2] * 12 + [3]),      # DPP kernel on chunks of 4096 + streamed radix 3
    (8192, [2] * 13),             # ... + one streamed radix-2 stage (kept dense in both directions)
    (28672, [2] * 12 + [7]),      # ... + streamed radix 7
    (14336, [2] * 11 + [7]),      # DPP kernel on chunks of 2048 + streamed radix 7
    (5120, [2] * 10 + [5]),       # DPP kernel on chunks of 1024 + streamed radix 5 (transposed: one launch)
    (6144, [2] * 11 + [3]),       # chunks of 2048, radix 3 (transposed: one launch)
    (10240, [2] * 11 + [5]),      # chunks of 2048, radix 5
    (7168, [2] * 10 + [7]),       # wave kernel on chunks of 1024 + streamed radix 7
    (2048 * 3, [2] * 9 + [4, 3]), # two streamed trips: halves on both sides of the first one
    (13824, [2] * 9 + [3, 3, 3]), # wave kernel on chunks of 512, two radix-3 stages in one trip, one more
])
def test_half_precision_intermediate_of_split_programs(harp, d, radices):
    """bf16 callers of a split program with one streamed small-radix stage: the intermediate
    travels as block-scaled halves (one power-of-two scale per 16 coordinates).  Rows chosen to
    stress that format -- zero rows, one-hot rows, rows 1e-30 and 1e18 in size (the two-shear form is specified for |x| < 2^64), a lone outlier of
    1e5 next to ordinary values, chunks of a row 1e12 apart in scale -- must still meet the bf16
    bar against the float64 oracle, in both directions; float32 callers keep float32."""
    import torch
    rng = np.random.default_rng(d)
    blocks = gi.make_blocks(d, radices, "orth", rng)
    signs = gi.make_signs(d, rng)
    plan = harp.Plan(d, radices, blocks, signs)
    name16, name32 = plan.kernel_name(64, harp.HARP_BF16), plan.kernel_name(64, harp.HARP_F32)
    say(f"half intermediate d={d} radices={radices}: bf16 -> {name16}, f32 -> {name32}")
    assert name16.endswith("_h16"), name16
    assert not name32.endswith("_h16"), name32
    g = rng.standard_normal
    rows = [np.zeros(d), np.eye(1, d, 5)[0], 3e4 * np.eye(1, d, d - 1)[0], 1e-30 * g(d), 1e18 * g(d)]
    r = g(d)
    r[d // 3] = 1e5
    rows.append(r)
    r = g(d) * np.where((np.arange(d) // 256) % 2 == 0, 1e6, 1e-6)
    rows.append(r)
    r = g(d)
    r[::16] *= 3e3                 # one large value in every segment of the input
    rows.append(r)
    X = np.concatenate([np.stack(rows), gi.activations(27, d, config=3, bf16=True).astype(np.float64)])
    X = gi.round_to_bf16(X.astype(np.float32))
    Yref = ho.apply_staged(X, d, radices, blocks, signs)
    Zref = ho.apply_transpose_staged(X, d, radices, blocks, signs)
    Y = to_host64(harp.harp_apply(plan, to_device(X, "bf16")))
    Z = to_host64(harp.harp_apply_transpose(plan, to_device(X, "bf16")))
    torch.cuda.synchronize()
    assert_parity(Y, Yref, "bf16", "apply")
    assert_parity(Z, Zref, "bf16", "apply_transpose")
    assert not Y[0].any() and not Z[0].any()       # a zero row stays exactly zero
    plan.destroy()
    # float32 intermediates on request
    pf = harp.Plan(d, radices, blocks, signs, flags=harp.HARP_F32_INTERMEDIATES)
    assert not pf.kernel_name(64, harp.HARP_BF16).endswith("_h16")
    assert_parity(to_host64(harp.harp_apply(pf, to_device(X, "bf16"))), Yref, "bf16", "apply, float32 intermediate")
    pf.destroy()


@pytest.mark.parametrize("d,radices", [(14336, [2] * 11 + [7]), (5120, [2] * 10 + [5]),
                                       (13824, [2] * 9 + [3, 3, 3]), (12288, [2] * 12 + [3]),
                                       (8192, [2] * 13)])
@pytest.mark.parametrize("n,ld_pad", [(0, 0), (1, 0), (2, 0), (3, 8), (5, 24), (67, 8), (6, 3)])
def test_half_precision_intermediate_edges(harp, d, radices, n, ld_pad):
    """Split programs of bf16 callers at the edges: no rows, one row, odd row counts (rows move in
    pairs), padded rows (the padding must not be written) and a padding that breaks the 16-byte
    alignment of the rows (the library must fall back to kernels that do not need it)."""
    run_case(harp, d, radices, n, "bf16", seed=d + 31 * n + ld_pad, ld_pad=ld_pad)


def test_half_precision_intermediate_in_place(harp):
    """harp_apply with Y == X on a split program whose intermediate travels as halves."""
    import torch
    d, radices, n = 14336, [2] * 11 + [7], 21
    rng = np.random.default_rng(5)
    blocks, signs = gi.make_blocks(d, radices, "orth", rng), gi.make_signs(d, rng)
    plan = harp.Plan(d, radices, blocks, signs)
    X = gi.round_to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    Xd = to_device(X, "bf16")
    harp.harp_apply(plan, Xd, Xd)
    torch.cuda.synchronize()
    assert_parity(to_host64(Xd), ho.apply_staged(X, d, radices, blocks, signs), "bf16", "apply in place")
    Xd = to_device(X, "bf16")
    harp.harp_apply_transpose(plan, Xd, Xd)
    torch.cuda.synchronize()
    assert_parity(to_host64(Xd), ho.apply_transpose_staged(X, d, radices, blocks, signs), "bf16",
                  "apply_transpose in place")
    plan.destroy()


def test_split_is_refused_when_there_is_nothing_to_split(harp):
    rng = np.random.default_rng(1)
    plan = harp.Plan(4096, [2] * 12, gi.make_blocks(4096, [2] * 12, "orth", rng))
    with pytest.raises(harp.HarpError) as e:
        plan.set_algo(harp.HARP_ALGO_SPLIT)
    assert e.value.status == harp.HARP_ERR_UNSUPPORTED
    plan.destroy()


@pytest.mark.parametrize("d,b,n,rows", [(12288, 3, 1, None), (12288, 3, 37, None), (20480, 5, 2, None),
                                        (20480, 5, 75, 6), (28672, 7, 5, None), (28672, 7, 130, None),
                                        (28672, 7, 33, 4), (12288, 3, 260, 2)])
def test_transposed_top_stage_fused_into_the_chunk_kernel(harp, d, b, n, rows):
    """Twelve radix-2 stages below one dense stage of radix 3 or 5, bf16, apply_transpose: one
    launch, the top stage executed while the rows are read (no float32 intermediate); ragged
    tiles, single rows, the two-launch fallbacks (in place, float32) and radix 7 (always two
    launches) alongside."""
    import torch
    radices = [2] * 12 + [b]
    X = gi.activations(n, d, config=3)
    run_case(harp, d, radices, n, "bf16", seed=d + n, rows=rows, act=X)
    if n == 37 or n == 5:
        rng = np.random.default_rng(d + n)
        blocks, signs = gi.make_blocks(d, radices, "orth", rng), gi.make_signs(d, rng)
        plan = harp.Plan(d, radices, blocks, signs)
        ref = ho.apply_transpose_staged(X, d, radices, blocks, signs)
        Xd = to_device(X, "bf16")
        harp.harp_apply_transpose(plan, Xd, Xd)                       # in place: two launches
        torch.cuda.synchronize()
        assert_parity(to_host64(Xd), ref, "bf16", "transpose in place")
        Xf = to_device(X, "f32")
        Zf = harp.harp_apply_transpose(plan, Xf)                      # float32: two launches
        torch.cuda.synchronize()
        assert_parity(to_host64(Zf), ref, "f32", "transpose float32")
        # generic (non-orthogonal) blocks through the fused launch
        plan.destroy()
        run_case(harp, d, radices, n, "bf16", kind="generic", seed=d + n + 1)


GENERIC_CASES = [
    # (d, radices, n, dtype): non-orthogonal blocks I + (0.3 / sqrt(b)) N(0,1) through every kernel family
    (4096, [2] * 12, 37, "bf16"), (4096, [2] * 12, 9, "f32"), (2048, [2] * 11, 21, "f32"),
    (1024, [2] * 10, 70, "bf16"), (256, [2] * 8, 33, "f32"), (4096, [8] * 4, 19, "f32"),
    (4096, [4] * 6, 11, "bf16"), (5120, [8, 8, 8, 5, 2], 13, "f32"), (11008, [2] * 8 + [43], 40, "bf16"),
    (11008, [2] * 8 + [43], 17, "f32"), (14336, [2] * 11 + [7], 24, "f32"), (13824, [2] * 9 + [3, 3, 3], 10, "bf16"),
    (1536, [2] * 9 + [3], 600, "f32"), (2752, [8, 8, 43], 30, "f32"), (120, [2, 3, 4, 5], 6, "f32"),
]


@pytest.mark.parametrize("d,radices,n,dtype", GENERIC_CASES)
def test_generic_non_orthogonal_blocks_through_every_kernel_family(harp, d, radices, n, dtype):
    """Blocks that are not orthogonal (max |K^T K - I| > 0.05): apply and apply_transpose are
    still the linear maps of the definition, to float32 rounding of the summands."""
    rng = np.random.default_rng(d + n)
    K = gi.make_blocks(d, radices, "generic", rng)
    assert max(float(np.abs(np.swapaxes(k, 1, 2).astype(np.float64) @ k - np.eye(k.shape[1])).max())
               for k in K) > 0.05
    run_case(harp, d, radices, n, dtype, kind="generic", seed=d + n)


def test_apply_never_blocks_and_never_frees_its_intermediate(harp):
    """A split program (float32 intermediate owned by the plan) called with 8 rows and then with
    2048 rows on one stream: neither call waits for the stream (both return while a long kernel
    queued ahead of them is still running), and both results match the oracle."""
    import torch
    d, radices = 14336, [2] * 11 + [7]
    rng = np.random.default_rng(21)
    blocks, signs = gi.make_blocks(d, radices, "orth", rng), gi.make_signs(d, rng)
    plan = harp.Plan(d, radices, blocks, signs)
    say("no host-side wait: n = 8 then n = 2048 on one stream", plan.kernel_name(2048))
    Xs = gi.round_to_bf16(rng.standard_normal((8, d)).astype(np.float32))
    Xl = gi.round_to_bf16(rng.standard_normal((2048, d)).astype(np.float32))
    Xsd, Xld = to_device(Xs, "bf16"), to_device(Xl, "bf16")
    Ys, Yl = torch.empty_like(Xsd), torch.empty_like(Xld)
    A = torch.randn(8192, 8192, device="cuda")
    torch.cuda.synchronize()
    st = torch.cuda.current_stream()
    done = torch.cuda.Event()
    for _ in range(12):                      # about 0.1 s of queued work ahead of the two calls
        A = (A @ A) * 1e-2
    harp.harp_apply(plan, Xsd, Ys, st)       # first call on the stream: allocates the small buffer
    harp.harp_apply(plan, Xld, Yl, st)       # needs the full slab: allocates again, frees nothing
    harp.harp_apply(plan, Xsd, Ys, st)
    done.record(st)
    returned_early = not done.query()
    torch.cuda.synchronize()
    assert returned_early, "harp_apply waited for the stream"
    assert_parity(to_host64(Ys), ho.apply_staged(Xs, d, radices, blocks, signs), "bf16", "n = 8")
    rows = np.arange(0, 2048, 16)
    assert_parity(to_host64(Yl)[rows], ho.apply_staged(Xl[rows], d, radices, blocks, signs), "bf16", "n = 2048")
    plan.destroy()


def test_graph_captured_at_small_n_survives_a_larger_eager_call(harp):
    """A graph captured with 8 rows holds the address of the plan's intermediate.  An eager call
    with 2048 rows on the same stream makes the plan take a larger one; the old buffer must stay
    alive, so that replaying the graph afterwards still gives the eager result."""
    import torch
    d, radices = 12288, [2] * 12 + [3]
    rng = np.random.default_rng(22)
    blocks, signs = gi.make_blocks(d, radices, "orth", rng), gi.make_signs(d, rng)
    plan = harp.Plan(d, radices, blocks, signs)
    say("graph at n = 8, then eager n = 2048, then replay", plan.kernel_name(8))
    Xs = gi.round_to_bf16(rng.standard_normal((8, d)).astype(np.float32))
    Xl = gi.round_to_bf16(rng.standard_normal((2048, d)).astype(np.float32))
    Xsd, Xld = to_device(Xs, "bf16"), to_device(Xl, "bf16")
    Yg, Yl = torch.zeros_like(Xsd), torch.empty_like(Xld)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        harp.harp_apply(plan, Xsd, Yg, side)          # warm-up on the capturing stream
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            harp.harp_apply(plan, Xsd, Yg, side)
        harp.harp_apply(plan, Xld, Yl, side)          # larger batch, same stream
        torch.cuda.synchronize()
        filler = [torch.full((1 << 22,), 3.0, device="cuda") for _ in range(8)]   # reuses freed memory, if any
    torch.cuda.current_stream().wait_stream(side)
    ref = ho.apply_staged(Xs, d, radices, blocks, signs)
    for rep in range(3):
        Yg.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_parity(to_host64(Yg), ref, "bf16", f"replay {rep} after the larger call")
        harp.harp_apply(plan, Xld, Yl, side)
        torch.cuda.synchronize()
    del filler
    rows = np.arange(0, 2048, 64)
    assert_parity(to_host64(Yl)[rows], ho.apply_staged(Xl[rows], d, radices, blocks, signs), "bf16", "n = 2048")
    plan.destroy()


@pytest.mark.parametrize("rows,cols,pad_in,pad_out,dtype", [(300, 4096, 8, 16, "bf16"), (33, 130, 0, 3, "f32"),
                                                           (1, 8, 0, 0, "bf16"), (2048, 4096, 0, 0, "bf16"),
                                                           (65, 1028, 4, 0, "f32"), (7, 24, 0, 8, "bf16")])
def test_identity_on_both_sides_is_a_plain_copy(harp, rows, cols, pad_in, pad_out, dtype):
    """rotate_weight with no processor on either side copies the matrix (16-byte pieces when rows
    and leading dimensions allow it, element by element otherwise) and leaves padding alone."""
    import torch
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    say("plain copy", rows, cols, pad_in, pad_out, dtype)
    src = torch.randn(rows, cols + pad_in, device="cuda").to(tdt)
    dst = torch.full((rows, cols + pad_out), 9.0, dtype=tdt, device="cuda")
    harp.harp_rotate_weight(None, None, src[:, :cols], dst[:, :cols])
    torch.cuda.synchronize()
    assert torch.equal(dst[:, :cols], src[:, :cols])
    if pad_out:
        assert bool((dst[:, cols:] == 9.0).all())


def test_rotate_weight_workspace_is_one_matrix_on_the_column_path(harp):
    rng = np.random.default_rng(2)
    pu = harp.Plan(64, [2] * 6, gi.make_blocks(64, [2] * 6, "orth", rng))
    pv = harp.Plan(48, [2, 2, 2, 2, 3], gi.make_blocks(48, [2, 2, 2, 2, 3], "orth", rng))
    pu11 = harp.Plan(44, [2, 2, 11], gi.make_blocks(44, [2, 2, 11], "orth", rng))
    mat = 64 * 48 * 4
    assert harp.harp_rotate_weight_workspace_size(pu, pv, 64, 48, harp.HARP_BF16) == mat
    assert harp.harp_rotate_weight_workspace_size(pu, None, 64, 48, harp.HARP_F32) == mat
    assert harp.harp_rotate_weight_workspace_size(None, pv, 64, 48, harp.HARP_F32) == 0
    # a radix above 8 on the U side: transposed-copy path, two float32 matrices with plan_V
    assert harp.harp_rotate_weight_workspace_size(pu11, pv, 44, 48, harp.HARP_F32) == 2 * 44 * 48 * 4
    for p in (pu, pv, pu11):
        p.destroy()


# ------------------------------------------------------------------ config 4: decode regime
@pytest.mark.parametrize("d,radices,n", [(4096, [2] * 12, 24), (14336, [2] * 11 + [7], 70)])
def test_graph_capture_and_replay(harp, d, radices, n):
    """The launches of an apply can be captured into a HIP graph (split programs after one
    eager call on the capturing stream, which allocates the plan's intermediate); every replay,
    with eager work and synchronisations in between, reproduces the eager result."""
    import torch
    rng = np.random.default_rng(d)
    blocks = gi.make_blocks(d, radices, "orth" if d == 4096 else "qr", rng)
    signs = gi.make_signs(d, rng)
    plan = harp.Plan(d, radices, blocks, signs)
    say(f"graph capture d={d} n={n} kernel={plan.kernel_name(n)}")
    X = gi.round_to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    Xd = to_device(X, "bf16")
    Y_eager = harp.harp_apply(plan, Xd).clone()
    Yg = torch.zeros_like(Xd)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        harp.harp_apply(plan, Xd, Yg, side)          # warm-up on the capturing stream
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            harp.harp_apply(plan, Xd, Yg, side)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        Yg.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Yg, Y_eager), f"replay {rep} differs from the eager result"
        other = harp.harp_apply_transpose(plan, Xd)   # eager work between replays
        torch.cuda.synchronize()
        assert other.shape == Xd.shape
    assert_parity(to_host64(Yg), ho.apply_staged(X, d, radices, blocks, signs), "bf16", "graph replay")
    plan.destroy()


def test_one_plan_on_two_streams_and_two_host_threads(harp):
    """A plan is immutable after create: two host threads drive it on two streams at the same
    time (a split program, whose float32 intermediate is kept per stream) and both reproduce the
    single-stream result bit for bit."""
    import threading
    import torch
    d, radices, n = 14336, [2] * 11 + [7], 300
    rng = np.random.default_rng(8)
    plan = harp.Plan(d, radices, gi.make_blocks(d, radices, "orth", rng), gi.make_signs(d, rng))
    Xs = [to_device(gi.round_to_bf16(rng.standard_normal((n, d)).astype(np.float32)), "bf16") for _ in range(2)]
    ref = [harp.harp_apply(plan, x).clone() for x in Xs]
    reft = [harp.harp_apply_transpose(plan, x).clone() for x in Xs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [[torch.zeros_like(Xs[i]), torch.zeros_like(Xs[i])] for i in range(2)]
    torch.cuda.synchronize()
    errors = []

    def worker(i):
        try:
            for rep in range(20):
                harp.harp_apply(plan, Xs[i], outs[i][0], stream=streams[i])
                harp.harp_apply_transpose(plan, Xs[i], outs[i][1], stream=streams[i])
            streams[i].synchronize()
        except Exception as e:  # noqa: BLE001
            errors.append(e)

    say("two streams, two host threads")
    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in range(2):
        assert torch.equal(outs[i][0], ref[i]) and torch.equal(outs[i][1], reft[i])
    plan.destroy()


def test_plan_from_theta_zero_is_the_randomized_hadamard_transform(harp):
    """Theta = 0, Hadamard mixers, power-of-two schedule: apply(x) = (x * sigma) H_d / sqrt(d),
    checked against scipy's Sylvester matrix, not against the staged oracle."""
    import torch
    from scipy.linalg import hadamard
    for d, radices in ((4096, [2] * 12), (4096, [8] * 4), (1024, [4, 2, 8, 16])):
        rng = np.random.default_rng(d + len(radices))
        signs = gi.make_signs(d, rng)
        plan = harp.Plan.from_theta(d, radices, None, None, signs)
        say(f"theta=0 d={d} radices={radices} kernel={plan.kernel_name(33)}")
        X = rng.standard_normal((33, d)).astype(np.float32)
        Y = to_host64(harp.harp_apply(plan, to_device(X, "f32")))
        Z = to_host64(harp.harp_apply_transpose(plan, to_device(X, "f32")))
        torch.cuda.synchronize()
        H = hadamard(d).astype(np.float64) / np.sqrt(d)
        assert_parity(Y, (X.astype(np.float64) * signs) @ H, "f32", "RHT apply")
        assert_parity(Z, (X.astype(np.float64) @ H.T) * signs, "f32", "RHT transpose")
        plan.destroy()


@pytest.mark.parametrize("d,radices,mixers", [
    (4096, [2] * 12, None), (4096, [8] * 4, None), (480, [2, 8, 3, 2, 5], "mixed"),
    (14336, [2] * 11 + [7], "odd_last")])
def test_plan_from_theta_matches_the_oracle_blocks(harp, d, radices, mixers):
    import torch
    rng = np.random.default_rng(d)
    thetas = [(0.8 * rng.standard_normal((d // b, b * (b - 1) // 2))).astype(np.float32) for b in radices]
    mix = None
    if mixers is not None:
        mix = []
        for b in radices:
            if b & (b - 1):      # the QR fallback of a seeded Gaussian (seed of the paper's unknown)
                q, r = np.linalg.qr(rng.standard_normal((b, b)))
                mix.append((q * np.sign(np.diag(r))).astype(np.float32))
            else:
                mix.append(None)
    signs = gi.make_signs(d, rng)
    plan = harp.Plan.from_theta(d, radices, thetas, mix, signs, flags=harp.HARP_VALIDATE_ORTHO)
    n = 21
    say(f"from theta d={d} radices={radices} kernel={plan.kernel_name(n)}")
    X = gi.round_to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    blocks = ho.blocks_from_theta(d, radices, thetas, mix)
    for dtype in ("f32", "bf16"):
        Y = to_host64(harp.harp_apply(plan, to_device(X, dtype)))
        Z = to_host64(harp.harp_apply_transpose(plan, to_device(X, dtype)))
        torch.cuda.synchronize()
        assert_parity(Y, ho.apply_staged(X, d, radices, blocks, signs), dtype, "apply")
        assert_parity(Z, ho.apply_transpose_staged(X, d, radices, blocks, signs), dtype, "apply_transpose")
    plan.destroy()


@pytest.mark.parametrize("d,radices", [(4096, [2] * 12), (4096, [8] * 4), (1680, [2, 8, 3, 5, 7])])
def test_plan_from_int8_theta(harp, d, radices):
    """Int8-stored parameters: the plan built from codes and scales applies the processor whose
    blocks the oracle rebuilds from the same codes (its own quantiser, dequantiser, Givens and
    Cayley maps)."""
    import torch
    rng = np.random.default_rng(d + len(radices))
    thetas = [(0.7 * rng.standard_normal((d // b, b * (b - 1) // 2))).astype(np.float32) for b in radices]
    mix = ["identity" if b & (b - 1) else None for b in radices]
    signs = gi.make_signs(d, rng)
    codes, scales = ho.quantize_theta_int8(d, radices, thetas)
    plan = harp.Plan.from_theta_int8(d, radices, codes, scales, mix, signs, flags=harp.HARP_VALIDATE_ORTHO)
    n = 19
    say(f"from int8 theta d={d} radices={radices} kernel={plan.kernel_name(n)}")
    X = gi.round_to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    blocks = ho.blocks_from_theta(d, radices, ho.dequantize_theta_int8(d, radices, codes, scales), mix)
    for dtype in ("f32", "bf16"):
        Y = to_host64(harp.harp_apply(plan, to_device(X, dtype)))
        Z = to_host64(harp.harp_apply_transpose(plan, to_device(X, dtype)))
        torch.cuda.synchronize()
        assert_parity(Y, ho.apply_staged(X, d, radices, blocks, signs), dtype, "apply")
        assert_parity(Z, ho.apply_transpose_staged(X, d, radices, blocks, signs), dtype, "apply_transpose")
    plan.destroy()


@pytest.mark.parametrize("d,radices,mix_kind,n,with_signs", [
    (4096, [8] * 4, None, 19, True),            # the default radix-8 schedule, Hadamard mixer
    (4096, [8] * 4, "identity", 8, False),
    (512, [8] * 3, None, 33, True),
    (1024, [4] * 5, None, 21, True),            # radix 4: six codes per block
    (256, [4] * 4, "identity", 5, True),
    (8192, [8] * 4 + [2], None, 37, True),      # chunk of 8^4 + one streamed radix-2 stage
    (5120, [8, 8, 8, 5, 2], "mixed", 9, True),  # no reconstructing kernel for this chunk: host blocks
])
def test_int8_theta_rebuilt_inside_the_kernel(harp, d, radices, mix_kind, n, with_signs):
    """HARP_THETA_IN_KERNEL: the chain kernel reads the int8 codes and rebuilds every block in
    registers (dequantise, Gauss-Jordan inverse of I + A, mixer, signs); the result is compared
    with the processor whose blocks the oracle rebuilds from the same codes in float64, and the
    plan without the flag (blocks rebuilt on the host) must give the same kernel family."""
    import torch
    rng = np.random.default_rng(d + 7 * len(radices) + n)
    thetas = [(0.5 * rng.standard_normal((d // b, b * (b - 1) // 2))).astype(np.float32) for b in radices]
    thetas[0][3] = 0.0                            # an all-zero block: scale 0, Q = I
    if mix_kind == "mixed":
        mix = ["identity" if b & (b - 1) else None for b in radices]
    else:
        mix = [mix_kind] * len(radices)
    signs = gi.make_signs(d, rng) if with_signs else None
    codes, scales = ho.quantize_theta_int8(d, radices, thetas)
    plan = harp.Plan.from_theta_int8(d, radices, codes, scales, mix, signs,
                                     flags=harp.HARP_VALIDATE_ORTHO | harp.HARP_THETA_IN_KERNEL)
    say(f"int8 theta in kernel d={d} radices={radices} mixers={mix_kind} kernel={plan.kernel_name(n)} "
        f"in_kernel={plan.theta_in_kernel()}")
    assert plan.theta_in_kernel()
    if mix_kind != "mixed":     # the reconstructing variant is the one that runs
        assert plan.kernel_name(n) in ("radix_tile_int8", "split_radix_stream_int8")
    else:
        assert not plan.kernel_name(n).endswith("_int8")
    X = gi.round_to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    blocks = ho.blocks_from_theta(d, radices, ho.dequantize_theta_int8(d, radices, codes, scales), mix)
    Yref = ho.apply_staged(X, d, radices, blocks, signs)
    Zref = ho.apply_transpose_staged(X, d, radices, blocks, signs)
    for dtype in ("f32", "bf16"):
        Y = to_host64(harp.harp_apply(plan, to_device(X, dtype)))
        Z = to_host64(harp.harp_apply_transpose(plan, to_device(X, dtype)))
        torch.cuda.synchronize()
        assert_parity(Y, Yref, dtype, "apply")
        assert_parity(Z, Zref, dtype, "apply_transpose")
    plan.destroy()


def test_kronecker_fallback_plan(harp):
    """d = 12 * 1024: T_d = (H~_12 / sqrt(12)) (x) T_1024 built by harp_kronecker_blocks."""
    import torch
    q = 11
    res = {(x * x) % q for x in range(1, q)}
    S = np.zeros((12, 12), dtype=np.int64)
    S[0, 1:] = 1
    S[1:, 0] = -1
    S[1:, 1:] = [[0 if i == j else (1 if ((i - j) % q) in res else -1) for j in range(q)] for i in range(q)]
    H12 = (np.eye(12, dtype=np.int64) + S).astype(np.float32)
    n2, radices2 = 1024, [2] * 10
    rng = np.random.default_rng(77)
    blocks2 = gi.make_blocks(n2, radices2, "orth", rng)
    radices, blocks = harp.harp_kronecker_blocks(H12, n2, radices2, blocks2)
    d = 12 * n2
    signs = gi.make_signs(d, rng)
    plan = harp.Plan(d, radices, blocks, signs)
    n = 19
    say(f"kronecker d={d} radices={radices} kernel={plan.kernel_name(n)}")
    X = gi.round_to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    Y = to_host64(harp.harp_apply(plan, to_device(X, "bf16")))
    torch.cuda.synchronize()
    # the definition: reshape to [K, n2], T_1024 along the last axis, H~/sqrt(K) across the first
    T2 = ho.build_U(n2, radices2, blocks2)
    Xs = (X.astype(np.float64) * signs).reshape(n, 12, n2)
    ref = np.einsum("nkj,kl,jm->nlm", Xs, H12.astype(np.float64) / np.sqrt(12.0), T2).reshape(n, d)
    assert_parity(Y, ref, "bf16", "kronecker apply")
    plan.destroy()


@pytest.mark.parametrize("K,n2,n,dtype,with_signs", [
    (12, 1024, 19, "bf16", True), (28, 512, 33, "f32", True), (20, 256, 70, "bf16", False),
    (28, 1024, 40, "bf16", True), (12, 1024, 5, "f32", False), (36, 256, 130, "bf16", True),
    (64, 512, 3, "f32", True)])
def test_kronecker_plan_with_tied_parameters(harp, K, n2, n, dtype, with_signs):
    """harp_plan_create_kronecker: one slice's parameters and one table on the device, read by
    every slice; apply and apply_transpose against the definition (H~/sqrt(K)) (x) T_{n2} with
    the signs on the input coordinates, and against the expanded (untied) plan."""
    import torch
    H = gi.hadamard_table(K)
    radices2 = [2] * int(np.log2(n2))
    rng = np.random.default_rng(K * n2 + n)
    blocks2 = gi.make_blocks(n2, radices2, "orth", rng)
    d = K * n2
    signs = gi.make_signs(d, rng) if with_signs else None
    plan = harp.Plan.kronecker(H, n2, radices2, blocks2, signs)
    radices, blocks = harp.harp_kronecker_blocks(H, n2, radices2, blocks2)
    full = harp.Plan(d, radices, blocks, signs)
    say(f"tied kronecker K={K} n2={n2} n={n} {dtype} signs={with_signs} kernel={plan.kernel_name(n)} "
        f"param bytes {plan.param_bytes()} vs {full.param_bytes()}")
    assert plan.tied_slices() == K and full.tied_slices() == 0
    assert plan.param_bytes() * (K // 2) < full.param_bytes()
    X = rng.standard_normal((n, d)).astype(np.float32)
    if dtype == "bf16":
        X = gi.round_to_bf16(X)
    Xd = to_device(X, dtype)
    Y, Z = harp.harp_apply(plan, Xd), harp.harp_apply_transpose(plan, Xd)
    Yf, Zf = harp.harp_apply(full, Xd), harp.harp_apply_transpose(full, Xd)
    torch.cuda.synchronize()
    T2 = ho.build_U(n2, radices2, blocks2)
    Hn = H.astype(np.float64) / np.sqrt(float(K))
    sg = np.ones(d) if signs is None else signs.astype(np.float64)
    X64 = X.astype(np.float64)
    ref = np.einsum("nkj,kl,jm->nlm", (X64 * sg).reshape(n, K, n2), Hn, T2).reshape(n, d)
    reft = np.einsum("nlm,kl,jm->nkj", X64.reshape(n, K, n2), Hn, T2).reshape(n, d) * sg
    assert_parity(to_host64(Y), ref, dtype, "tied apply")
    assert_parity(to_host64(Z), reft, dtype, "tied apply_transpose")
    assert_parity(to_host64(Yf), ref, dtype, "expanded apply")
    assert_parity(to_host64(Zf), reft, dtype, "expanded apply_transpose")
    # padded leading dimension (a multiple of 8) and in place
    big = torch.zeros(n, d + 16, dtype=Xd.dtype, device="cuda")
    big[:, :d] = Xd
    harp.harp_apply(plan, big[:, :d], big[:, :d])
    torch.cuda.synchronize()
    assert_parity(to_host64(big[:, :d]), ref, dtype, "tied apply in place, padded")
    assert bool((big[:, d:] == 0).all())
    plan.destroy()
    full.destroy()


def test_kronecker_plan_falls_back_to_the_expansion_and_refuses_unaligned_rows(harp):
    import torch
    rng = np.random.default_rng(5)
    # a table of order 4 (below 9) and slices with a radix other than 2: no tied kernel, same results
    for K, n2, radices2 in ((4, 1024, [2] * 10), (12, 192, [4, 6, 8])):
        H = gi.hadamard_table(K)
        blocks2 = gi.make_blocks(n2, radices2, "orth", rng)
        d = K * n2
        signs = gi.make_signs(d, rng)
        plan = harp.Plan.kronecker(H, n2, radices2, blocks2, signs)
        assert plan.tied_slices() == 0
        X = gi.round_to_bf16(rng.standard_normal((7, d)).astype(np.float32))
        Y = to_host64(harp.harp_apply(plan, to_device(X, "bf16")))
        torch.cuda.synchronize()
        T2 = ho.build_U(n2, radices2, blocks2)
        ref = np.einsum("nkj,kl,jm->nlm", (X.astype(np.float64) * signs).reshape(7, K, n2),
                        H.astype(np.float64) / np.sqrt(float(K)), T2).reshape(7, d)
        assert_parity(Y, ref, "bf16", "fallback apply")
        plan.destroy()
    # tied plan: rows that are not 16-byte aligned are refused, not mis-read
    H = gi.hadamard_table(12)
    blocks2 = gi.make_blocks(256, [2] * 8, "orth", rng)
    plan = harp.Plan.kronecker(H, 256, [2] * 8, blocks2, None)
    assert plan.tied_slices() == 12
    big = torch.zeros(4, 12 * 256 + 3, dtype=torch.float32, device="cuda")
    with pytest.raises(harp.HarpError) as e:
        harp.harp_apply(plan, big[:, 1:1 + 12 * 256])
    assert e.value.status == harp.HARP_ERR_UNSUPPORTED
    with pytest.raises(harp.HarpError) as e:
        plan.set_algo(harp.HARP_ALGO_FUSED)
    assert e.value.status == harp.HARP_ERR_UNSUPPORTED
    # as the row-side processor of a weight rotation
    W = rng.standard_normal((24, 12 * 256)).astype(np.float32)
    pu = harp.Plan(24, [2, 3, 4], gi.make_blocks(24, [2, 3, 4], "orth", rng))
    out = harp.harp_rotate_weight(pu, plan, to_device(W, "f32"))
    torch.cuda.synchronize()
    T2 = ho.build_U(256, [2] * 8, blocks2)
    Uu = ho.build_U(24, [2, 3, 4], gi.make_blocks(24, [2, 3, 4], "orth", np.random.default_rng(0)))
    del Uu
    radices, blocks = harp.harp_kronecker_blocks(H, 256, [2] * 8, blocks2)
    full = harp.Plan(12 * 256, radices, blocks, None)
    ref = harp.harp_rotate_weight(pu, full, to_device(W, "f32"))
    torch.cuda.synchronize()
    assert float((out - ref).abs().max()) <= 2e-6 * float(ref.abs().max())
    for p_ in (plan, full, pu):
        p_.destroy()


RADIX_TILE_CASES = [
    (512, [8] * 3, 19), (4096, [8] * 4, 37), (4096, [8] * 4, 1), (256, [4] * 4, 9), (1024, [4] * 5, 21),
    (4096, [4] * 6, 13), (4096, [8] * 4, 8),
]


@pytest.mark.parametrize("d,radices,n", RADIX_TILE_CASES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_equal_small_radix_tile_kernel(harp, d, radices, n, dtype):
    """All stages radix 4 or all radix 8: the tile kernel with prefetched block parameters."""
    blocks = gi.make_blocks(d, radices, "qr", np.random.default_rng(1))
    plan = harp.Plan(d, radices, blocks, None)
    assert plan.kernel_name(n) == "radix_tile", plan.kernel_name(n)
    plan.destroy()
    run_case(harp, d, radices, n, dtype, kind="qr", seed=d + n)
    run_case(harp, d, radices, n, dtype, kind="orth", seed=d + n + 1, ld_pad=8, with_signs=False)
    run_case(harp, d, radices, n, dtype, kind="qr", seed=d + n + 2, ld_pad=3)   # unaligned: fallback


@pytest.mark.parametrize("d,radices,n", [(28672, [8, 8, 8, 8, 7], 70), (768, [4, 4, 4, 4, 3], 65),
                                         (5120, [8, 8, 8, 5, 2], 66)])
def test_split_program_with_small_radix_chunk(harp, d, radices, n):
    run_case(harp, d, radices, n, "bf16", kind="qr", seed=d)


MIXED_RADIX_CASES = [
    (3584, [8, 8, 8, 7], 19), (2560, [8, 8, 8, 5], 9), (14336, [8, 8, 8, 7, 4], 37), (5120, [8, 8, 8, 5, 2], 21),
    (1344, [8, 8, 7, 3], 5), (960, [4, 8, 5, 6], 13), (11008, [8, 8, 4, 43], 11),
]


@pytest.mark.parametrize("d,radices,n", MIXED_RADIX_CASES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_mixed_small_radix_tile_kernel(harp, d, radices, n, dtype):
    """Chunks whose stages have different radices in 3..8 (the paper's greedy schedules)."""
    run_case(harp, d, radices, n, dtype, kind="qr", seed=d + n)
    run_case(harp, d, radices, n, dtype, kind="qr", seed=d + n + 1, ld_pad=8, rows=3)


def test_radix_tile_kernel_in_place(harp):
    import torch
    d, radices, n = 4096, [8] * 4, 11
    rng = np.random.default_rng(12)
    blocks = gi.make_blocks(d, radices, "qr", rng)
    signs = gi.make_signs(d, rng)
    X = gi.round_to_bf16(rng.standard_normal((n, d)).astype(np.float32))
    plan = harp.Plan(d, radices, blocks, signs)
    say("radix tile in place", plan.kernel_name(n))
    Xd = to_device(X, "bf16")
    harp.harp_apply(plan, Xd, Xd)
    torch.cuda.synchronize()
    assert_parity(to_host64(Xd), ho.apply_staged(X, d, radices, blocks, signs), "bf16", "apply in place")
    plan.destroy()


@pytest.mark.parametrize("n", [1, 8, 32, 64])
@pytest.mark.parametrize("d,radices", [(4096, [2] * 12), (12288, [2] * 12 + [3]), (14336, [2] * 11 + [7])])
def test_decode_regime(harp, n, d, radices):
    X = gi.activations(n, d, config=4, dist="normal", outlier_frac=0.005, outlier_scale=50.0)
    run_case(harp, d, radices, n, "bf16", seed=4000 + d + n, act=X, both=False)


# ------------------------------------------------------------------ config 5: d = 28672, 8192
def test_full_size_28672(harp):
    """4096 x 28672: one row out of every four consecutive ones (1024 rows), both directions; the
    row tiles of every launch of this shape hold more than four rows."""
    _full_size(harp, "ffn70b_28672_r2x12_7", row_step=4)


def test_radix2_chain_8192(harp):
    run_case(harp, 8192, [2] * 13, 40, "bf16", seed=13, act=gi.activations(40, 8192, config=5))


# ------------------------------------------------------------------ rotate_weight
def _plan_tuple(d, radices, blocks, signs):
    return (d, radices, blocks, signs)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("do,ru,di,rv", [(24, [2, 3, 4], 40, [8, 5]), (64, [2] * 6, 48, [2, 2, 2, 2, 3]),
                                         (14, [2, 7], 30, [2, 3, 5]), (192, [4, 6, 8], 130, [2, 5, 13]),
                                         (256, [2] * 8, 344, [2, 2, 2, 43]),
                                         # plan_U in column mode: two passes, odd column count
                                         (512, [2] * 9, 65, [5, 13]), (1024, [2] * 10, 96, [2] * 5 + [3]),
                                         (240, [5, 6, 8], 34, [2, 17]), (96, [3, 2, 2, 2, 4], 130, [130 // 13, 13]),
                                         (384, [2, 2, 3, 2, 2, 2, 2, 2], 258, [2, 3, 43]),
                                         # plan_U with a radix above 8: transposed-copy path
                                         (44, [2, 2, 11], 24, [2, 3, 4]),
                                         # column passes whose tile height is not 32 / 64 / 128
                                         # (28, 27, 21, 48 rows): unguarded kernel with repeated rows
                                         (896, [2] * 7 + [7], 256, [2] * 8),
                                         (1728, [8, 8, 3, 3, 3], 128, [2] * 7),
                                         (1344, [7, 3, 8, 8], 384, [2] * 7 + [3]),
                                         (1536, [3] + [2] * 9, 130, [2, 5, 13])])
def test_rotate_weight_small_dense(harp, dtype, do, ru, di, rv):
    import torch
    rng = np.random.default_rng(do + di)
    bu, bv = gi.make_blocks(do, ru, "orth", rng), gi.make_blocks(di, rv, "orth", rng)
    su, sv = gi.make_signs(do, rng), gi.make_signs(di, rng)
    W = rng.standard_normal((do, di)).astype(np.float32)
    if dtype == "bf16":
        W = gi.round_to_bf16(W)
    pu, pv = harp.Plan(do, ru, bu, su), harp.Plan(di, rv, bv, sv)
    say("rotate_weight", do, di, dtype)
    Wd = to_device(W, dtype)
    ref = ho.rotate_weight(W, _plan_tuple(do, ru, bu, su), _plan_tuple(di, rv, bv, sv))
    out = harp.harp_rotate_weight(pu, pv, Wd)
    torch.cuda.synchronize()
    assert_parity(to_host64(out), ref, dtype, "U^T W V")
    # one-sided
    assert_parity(to_host64(harp.harp_rotate_weight(None, pv, Wd)),
                  ho.rotate_weight(W, None, _plan_tuple(di, rv, bv, sv)), dtype, "W V")
    assert_parity(to_host64(harp.harp_rotate_weight(pu, None, Wd)),
                  ho.rotate_weight(W, _plan_tuple(do, ru, bu, su), None), dtype, "U^T W")
    assert torch.equal(harp.harp_rotate_weight(None, None, Wd), Wd)
    # inverse map on the float64-exact input: U (U^T W V) V^T = W
    Uu, Uv = ho.build_U(do, ru, bu, su), ho.build_U(di, rv, bv, sv)
    inv = to_host64(harp.harp_rotate_weight_inverse(pu, pv, Wd))
    assert_parity(inv, Uu @ W.astype(np.float64) @ Uv.T, dtype, "U W V^T")
    # in place
    W2 = Wd.clone()
    harp.harp_rotate_weight(pu, pv, W2, W2)
    torch.cuda.synchronize()
    assert torch.equal(W2, out)
    pu.destroy()
    pv.destroy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rotate_weight_views_with_padding_and_odd_offsets(harp, dtype):
    """Matrices that are views into wider buffers (leading dimension above d_in, first element
    at an odd offset): the column-mode passes then take their element-by-element path."""
    import torch
    do, ru, di, rv = 256, [2] * 8, 70, [2, 5, 7]
    rng = np.random.default_rng(77)
    bu, bv = gi.make_blocks(do, ru, "orth", rng), gi.make_blocks(di, rv, "orth", rng)
    su, sv = gi.make_signs(do, rng), gi.make_signs(di, rng)
    W = rng.standard_normal((do, di)).astype(np.float32)
    if dtype == "bf16":
        W = gi.round_to_bf16(W)
    pu, pv = harp.Plan(do, ru, bu, su), harp.Plan(di, rv, bv, sv)
    ref = ho.rotate_weight(W, _plan_tuple(do, ru, bu, su), _plan_tuple(di, rv, bv, sv))
    ref_u = ho.rotate_weight(W, _plan_tuple(do, ru, bu, su), None)
    Wd = to_device(W, dtype)
    for pad, off in [(3, 1), (2, 0), (9, 5)]:
        say("rotate_weight view", dtype, pad, off)
        big_in = torch.zeros(do, di + pad + off, dtype=Wd.dtype, device="cuda")
        big_out = torch.full((do, di + pad + off), 7.0, dtype=Wd.dtype, device="cuda")
        vin, vout = big_in[:, off:off + di], big_out[:, off:off + di]
        vin.copy_(Wd)
        harp.harp_rotate_weight(pu, pv, vin, vout)
        torch.cuda.synchronize()
        assert_parity(to_host64(vout.contiguous()), ref, dtype, "U^T W V (view)")
        harp.harp_rotate_weight(pu, None, vin, vout)
        torch.cuda.synchronize()
        assert_parity(to_host64(vout.contiguous()), ref_u, dtype, "U^T W (view)")
        # nothing outside the view is written
        assert bool((big_out[:, :off] == 7.0).all()) and bool((big_out[:, off + di:] == 7.0).all())
    pu.destroy()
    pv.destroy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("do,ru,di,rv", [
    (64, [2] * 6, 12288, [2] * 12 + [3]),            # one column pass of 64 rows, radix-3 row stage
    (32, [4, 8], 20480, [2] * 12 + [5]),             # 32 rows, radix 5
    (4096, [2] * 12, 28672, [2] * 12 + [7]),         # two column passes (128 + 32 rows), radix 7
    (192, [3, 8, 8], 8192 * 3, [2] * 13 + [3])])     # passes of 24 and 8 rows: not fusable
def test_rotate_weight_with_streamed_row_stage(harp, dtype, do, ru, di, rv):
    """plan_V longer than one on-chip chunk with a small-radix top stage: that stage is executed
    inside one of plan_U's column passes.  Rows of the result are recomputed by the oracle."""
    import torch
    rng = np.random.default_rng(do + di)
    bu, bv = gi.make_blocks(do, ru, "orth", rng), gi.make_blocks(di, rv, "orth", rng)
    su, sv = gi.make_signs(do, rng), gi.make_signs(di, rng)
    W = (rng.standard_normal((do, di)) * 0.1).astype(np.float32)
    if dtype == "bf16":
        W = gi.round_to_bf16(W)
    pu, pv = harp.Plan(do, ru, bu, su), harp.Plan(di, rv, bv, sv)
    say("rotate_weight with streamed row stage", do, di, dtype)
    Wd = to_device(W, dtype)
    out = harp.harp_rotate_weight(pu, pv, Wd)
    inv = harp.harp_rotate_weight_inverse(pu, pv, Wd)
    torch.cuda.synchronize()
    rows = sorted(set([0, 1, do // 3, do - 1]))
    E = np.zeros((len(rows), do))
    E[np.arange(len(rows)), rows] = 1.0
    W64 = W.astype(np.float64)
    # row i of U^T W V = (e_i U^T) W V;  row i of U W V^T = (e_i U) W V^T
    ref = ho.apply_staged(ho.apply_transpose_staged(E, do, ru, bu, su) @ W64, di, rv, bv, sv)
    refi = ho.apply_transpose_staged(ho.apply_staged(E, do, ru, bu, su) @ W64, di, rv, bv, sv)
    idx = torch.tensor(rows).cuda()
    assert_parity(to_host64(out[idx]), ref, dtype, "U^T W V rows")
    assert_parity(to_host64(inv[idx]), refi, dtype, "U W V^T rows")
    # in place, and round trip back to W
    W2 = Wd.clone()
    harp.harp_rotate_weight(pu, pv, W2, W2)
    torch.cuda.synchronize()
    assert torch.equal(W2, out)
    back = harp.harp_rotate_weight_inverse(pu, pv, out)
    torch.cuda.synchronize()
    err = float((back.float() - Wd.float()).abs().max()) / float(Wd.float().abs().max())
    assert err < (2e-2 if dtype == "bf16" else 1e-4), err
    pu.destroy()
    pv.destroy()


@pytest.mark.parametrize("do,ru,di,rv", [
    (1024, [2] * 10, 4096, [2] * 12),        # two column passes; plan_V in one launch (4096)
    (2048, [8, 8, 8, 4], 2048, [2] * 11),    # radix-8 column passes; plan_V on 2048 coordinates
    (256, [2] * 8, 1024, [2] * 10),          # plan_V on 1024 coordinates
    (128, [2] * 7, 4096, [2] * 12),          # one column pass of 128 rows (bf16 -> bf16 when one-sided)
    (32, [2] * 5, 2048, [2] * 11),           # ... of 32 rows
    (896, [2] * 7 + [7], 14336, [2] * 11 + [7]),   # row stage fused into a column pass
    (448, [2] * 6 + [7], 8192, [2] * 13),          # plan_V with a radix-2 stage on its top digit: own trip
    (640, [2] * 7 + [5], 5120, [2] * 10 + [5])])
def test_rotate_weight_half_precision_workspace(harp, do, ru, di, rv):
    """bf16 matrices between orthogonal processors travel through the workspace as block-scaled
    halves: both maps, one-sided calls and in place, rows recomputed by the oracle."""
    import torch
    rng = np.random.default_rng(do * 7 + di)
    bu, bv = gi.make_blocks(do, ru, "orth", rng), gi.make_blocks(di, rv, "orth", rng)
    su, sv = gi.make_signs(do, rng), gi.make_signs(di, rng)
    # heavy-tailed entries with a few large columns and rows
    W = rng.standard_t(3, size=(do, di)) * 0.02
    W[:, rng.choice(di, 5, replace=False)] *= 20.0
    W[rng.choice(do, 3, replace=False), :] *= 8.0
    W = gi.round_to_bf16(W.astype(np.float32))
    pu, pv = harp.Plan(do, ru, bu, su), harp.Plan(di, rv, bv, sv)
    say("rotate_weight, half-precision workspace", do, di)
    Wd = to_device(W, "bf16")
    out = harp.harp_rotate_weight(pu, pv, Wd)
    inv = harp.harp_rotate_weight_inverse(pu, pv, Wd)
    out_u = harp.harp_rotate_weight(pu, None, Wd)
    inv_u = harp.harp_rotate_weight_inverse(pu, None, Wd)
    torch.cuda.synchronize()
    step = max(1, do // 37)
    rows = sorted(set(list(range(0, do, step)) + [1, do - 1]))
    E = np.zeros((len(rows), do))
    E[np.arange(len(rows)), rows] = 1.0
    W64 = W.astype(np.float64)
    UtW = ho.apply_transpose_staged(E, do, ru, bu, su) @ W64     # rows of U^T W
    UW = ho.apply_staged(E, do, ru, bu, su) @ W64                # rows of U W
    idx = torch.tensor(rows).cuda()
    assert_parity(to_host64(out[idx]), ho.apply_staged(UtW, di, rv, bv, sv), "bf16", "U^T W V rows")
    assert_parity(to_host64(inv[idx]), ho.apply_transpose_staged(UW, di, rv, bv, sv), "bf16", "U W V^T rows")
    # one-sided: plan_U transforms the columns of W, and the bar's scale floor is the column's
    # (with columns 20 times the others a row's scale says nothing about the entries of that
    # column; between the launches an entry carries 2^-12 of itself)
    colscale = np.linalg.norm(W64, axis=0, keepdims=True) / np.sqrt(do)
    assert_parity(to_host64(out_u[idx]), UtW, "bf16", "U^T W rows", rho=colscale)
    assert_parity(to_host64(inv_u[idx]), UW, "bf16", "U W rows", rho=colscale)
    # float32 intermediates on request: the one-sided result then meets the bar with the row's
    # scale as well
    pf = harp.Plan(do, ru, bu, su, flags=harp.HARP_F32_INTERMEDIATES)
    out_f = harp.harp_rotate_weight(pf, None, Wd)
    torch.cuda.synchronize()
    assert_parity(to_host64(out_f[idx]), UtW, "bf16", "U^T W rows, float32 workspace")
    pf.destroy()
    # the Frobenius norm is preserved
    nw = float(torch.linalg.matrix_norm(Wd.float()))
    for t in (out, inv, out_u, inv_u):
        assert abs(float(torch.linalg.matrix_norm(t.float())) - nw) / nw < 2e-3
    # in place
    W2 = Wd.clone()
    harp.harp_rotate_weight(pu, pv, W2, W2)
    W3 = Wd.clone()
    harp.harp_rotate_weight_inverse(pu, None, W3, W3)
    torch.cuda.synchronize()
    assert torch.equal(W2, out) and torch.equal(W3, inv_u)
    pu.destroy()
    pv.destroy()


def test_rotate_weight_llama70b_shape_sampled(harp):
    """W 8192 x 28672 bf16: rows of U^T W V recomputed one by one by the oracle."""
    import torch
    do, di = 8192, 28672
    ru, rv = [2] * 13, [2] * 12 + [7]
    bu, su = gi.processor(do, ru, config=5, salt=1)
    bv, sv = gi.processor(di, rv, config=5, salt=2)
    W = gi.weights(do, di, config=5)
    pu, pv = harp.Plan(do, ru, bu, su), harp.Plan(di, rv, bv, sv)
    say("rotate_weight 8192x28672 bf16")
    Wd = to_device(W, "bf16")
    out = harp.harp_rotate_weight(pu, pv, Wd)
    torch.cuda.synchronize()
    # 256 rows: one in every band of 32 consecutive rows (the row tiles of plan_V's chunk kernel
    # and the 128-row tiles of the first column pass), hitting every residue modulo 128 (the
    # tiles of the second column pass, rows lo + 128 j); whole rows, so every column tile too
    k = np.arange(256)
    rows = 32 * k + (29 * (k // 4) + 5 * (k % 4)) % 32
    assert len(set(rows % 128)) == 128 and len(set(rows // 32)) == 256
    rows = [int(r) for r in rows]
    E = np.zeros((len(rows), do))
    E[np.arange(len(rows)), rows] = 1.0
    # row i of U^T is e_i U^T
    UtW = ho.apply_transpose_staged(E, do, ru, bu, su) @ W.astype(np.float64)
    ref = ho.apply_staged(UtW, di, rv, bv, sv)
    got = to_host64(out[torch.tensor(rows).cuda()])
    assert_parity(got, ref, "bf16", "rotate_weight rows")
    # Frobenius norm is preserved
    nw = float(torch.linalg.matrix_norm(Wd.float()))
    no = float(torch.linalg.matrix_norm(out.float()))
    assert abs(no - nw) / nw < 1e-3
    pu.destroy()
    pv.destroy()


def test_rotate_weight_llama70b_gate_shape_sampled(harp):
    """W 28672 x 8192 bf16 (the transposed 70B shape): plan_U with a radix-7 stage among its column
    passes, plan_V = 2^13 whose top stage takes its own trip; rows recomputed by the oracle, both maps."""
    import torch
    do, di = 28672, 8192
    ru, rv = [2] * 12 + [7], [2] * 13
    bu, su = gi.processor(do, ru, config=5, salt=3)
    bv, sv = gi.processor(di, rv, config=5, salt=4)
    W = gi.weights(do, di, config=5)
    pu, pv = harp.Plan(do, ru, bu, su), harp.Plan(di, rv, bv, sv)
    say("rotate_weight 28672x8192 bf16")
    Wd = to_device(W, "bf16")
    out = harp.harp_rotate_weight(pu, pv, Wd)
    inv = harp.harp_rotate_weight_inverse(pu, pv, Wd)
    torch.cuda.synchronize()
    k = np.arange(96)
    rows = [int(r) for r in (298 * k + 7 * (k % 13)) % do]
    rows = sorted(set(rows + [0, do - 1]))
    E = np.zeros((len(rows), do))
    E[np.arange(len(rows)), rows] = 1.0
    W64 = W.astype(np.float64)
    ref = ho.apply_staged(ho.apply_transpose_staged(E, do, ru, bu, su) @ W64, di, rv, bv, sv)
    refi = ho.apply_transpose_staged(ho.apply_staged(E, do, ru, bu, su) @ W64, di, rv, bv, sv)
    idx = torch.tensor(rows).cuda()
    assert_parity(to_host64(out[idx]), ref, "bf16", "U^T W V rows")
    assert_parity(to_host64(inv[idx]), refi, "bf16", "U W V^T rows")
    nw = float(torch.linalg.matrix_norm(Wd.float()))
    for t in (out, inv):
        assert abs(float(torch.linalg.matrix_norm(t.float())) - nw) / nw < 1e-3
    pu.destroy()
    pv.destroy()
