"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test is chosen so that a plausible mistake in oracle/harp_oracle.py -- a wrong
stride, a transposed block, a swapped block index, reversed stage order, misplaced
signs -- fails at least one of them.
"""
import os

import numpy as np
import pytest
import scipy.linalg

from oracle import harp_oracle as ho
from paper_2605_29843_amd import inputs as gi

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_golden(name):
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split(":")
                rows.append((k.strip(), v.strip()))
    return rows


def _rand_blocks(d, radices, seed, orth=True):
    rng = np.random.default_rng(seed)
    if orth:
        return gi.make_blocks(d, radices, "qr", rng)      # non-symmetric, det = +-1
    return [rng.standard_normal((d // b, b, b)).astype(np.float32) for b in radices]


# ------------------------------------------------------------------ index convention
def test_index_example_d16_b4():
    """Appendix index-view example: which coordinates each stage's blocks mix."""
    gold = {int(k): [[int(x) for x in grp.split()] for grp in v.split("|")]
            for k, v in _read_golden("index_example_d16_b4.txt")}
    d, radices = 16, [4, 4]
    st = ho.strides(radices)
    for t in (0, 1):
        # block c mixes exactly the support of the rows of the stage matrix in its group
        for c in range(4):
            K = np.tile(np.eye(4), (4, 1, 1))
            K[c] = np.full((4, 4), 1.0)              # block c couples all its coordinates
            Y = np.eye(d)
            ho.stage_apply_rows(Y, 4, st[t], K)
            coupled = sorted(np.nonzero((Y - np.eye(d)).any(axis=0))[0].tolist())
            assert coupled in gold[t], (t, c, coupled)
        # and the blocks are numbered c = alpha*s + beta: stage 0 -> group c is 4c..4c+3;
        # stage 1 -> group c is c, c+4, c+8, c+12
        for c in range(4):
            K = np.tile(np.eye(4), (4, 1, 1))
            K[c] = np.full((4, 4), 1.0)
            Y = np.eye(d)
            ho.stage_apply_rows(Y, 4, st[t], K)
            coupled = sorted(np.nonzero((Y - np.eye(d)).any(axis=0))[0].tolist())
            assert coupled == gold[t][c]


def test_strides_and_schedule_check():
    assert ho.strides([8, 8, 4, 43]) == [1, 8, 64, 256]
    ho.check_schedule(11008, [2] * 8 + [43])
    with pytest.raises(ValueError):
        ho.check_schedule(16, [4, 2])
    with pytest.raises(ValueError):
        ho.check_schedule(16, [16, 1])
    with pytest.raises(ValueError):
        ho.check_schedule(4, [])


# ------------------------------------------------------------------ one stage = Kronecker form
@pytest.mark.parametrize("g,b,s", [(1, 4, 1), (3, 2, 4), (2, 3, 5), (4, 5, 2), (1, 7, 6), (5, 8, 1)])
def test_stage_equals_kron_when_blocks_equal(g, b, s):
    """Lemma 1: with one shared block K the stage is x (I_g kron K kron I_s).

    K is non-symmetric, so a transposed block multiply fails here."""
    d = g * b * s
    rng = np.random.default_rng(7 + d)
    K1 = rng.standard_normal((b, b))
    K = np.broadcast_to(K1, (d // b, b, b)).copy()
    X = rng.standard_normal((5, d))
    Y = ho.stage_apply_rows(X.copy(), b, s, K)
    M = np.kron(np.kron(np.eye(g), K1), np.eye(s))
    np.testing.assert_allclose(Y, X @ M, rtol=0, atol=1e-13)
    Yt = ho.stage_apply_rows(X.copy(), b, s, K, transpose_blocks=True)
    np.testing.assert_allclose(Yt, X @ M.T, rtol=0, atol=1e-13)


def test_stage_block_numbering_alpha_major():
    """Block c = alpha*s + beta: scale block c by (c+1) and read the scaling back."""
    g, b, s = 3, 2, 4
    d = g * b * s
    K = np.stack([np.eye(b) * (c + 1) for c in range(d // b)])
    y = ho.stage_apply_rows(np.ones((1, d)), b, s, K)[0]
    for alpha in range(g):
        for r in range(b):
            for beta in range(s):
                assert y[alpha * b * s + r * s + beta] == alpha * s + beta + 1


# ------------------------------------------------------------------ Theta = 0  ==>  RHT
@pytest.mark.parametrize("radices", [[2] * 6, [8, 8, 4], [4, 2, 8], [16, 4], [2] * 8, [8, 8, 8, 8]])
def test_theta_zero_is_normalised_sylvester_hadamard(radices):
    """Theorem 1 / Lemmas 1-2: all blocks = H_b gives the Walsh-Hadamard transform.
    Under the Lemma-1 flattening the fixed permutation is the identity, so the dense U
    must equal scipy's Sylvester matrix / sqrt(d)."""
    d = int(np.prod(radices))
    blocks = gi.make_blocks(d, radices, "hadamard", None)
    U = ho.build_U(d, radices, blocks)
    H = scipy.linalg.hadamard(d) / np.sqrt(d)
    assert np.max(np.abs(U - H)) < 1e-6          # blocks are float32 values
    # exact-in-float64 blocks: deviation at rounding level
    blocks64 = [np.broadcast_to(ho.sylvester_hadamard(b), (d // b, b, b)).copy() for b in radices]
    U64 = ho.build_U(d, radices, blocks64)
    assert np.max(np.abs(U64 - H)) < 1e-14
    # closed form (-1)^{popcount(i & j)} / sqrt(d)
    i = np.arange(d)
    pc = np.vectorize(lambda v: bin(v).count("1"))(i[:, None] & i[None, :])
    np.testing.assert_allclose(U64, (-1.0) ** pc / np.sqrt(d), atol=1e-14)


def test_rht_with_signs_is_diag_sigma_times_hadamard():
    d, radices = 64, [2] * 6
    blocks = [np.broadcast_to(ho.sylvester_hadamard(2), (d // 2, 2, 2)).copy() for _ in radices]
    sg = gi.make_signs(d, np.random.default_rng(3))
    U = ho.build_U(d, radices, blocks, sg)
    H = scipy.linalg.hadamard(d) / np.sqrt(d)
    np.testing.assert_allclose(U, np.diag(sg.astype(float)) @ H, atol=1e-14)


def test_sylvester_recursion_and_orthogonality():
    for b in (1, 2, 4, 8, 16, 32):
        H = ho.sylvester_hadamard(b)
        np.testing.assert_allclose(H.T @ H, np.eye(b), atol=1e-14)
        np.testing.assert_allclose(H * np.sqrt(b), scipy.linalg.hadamard(b), atol=1e-14)


# ------------------------------------------------------------------ orthogonality / round trip
SCHEDULES = [[2, 2, 2], [4, 4], [2, 3], [3, 2], [8, 5], [2, 2, 7], [5, 2, 3], [2] * 8,
             [8, 8, 4], [2, 2, 2, 3], [4, 43]]


@pytest.mark.parametrize("radices", SCHEDULES)
def test_orthogonality_norm_roundtrip(radices):
    d = int(np.prod(radices))
    rng = np.random.default_rng(d)
    # float64 orthogonal blocks so the 1e-12 bound is about the oracle, not float32 inputs
    blocks = []
    for b in radices:
        Q, R = np.linalg.qr(rng.standard_normal((d // b, b, b)))
        blocks.append(Q)
    sg = gi.make_signs(d, rng)
    U = ho.build_U(d, radices, blocks, sg)
    assert np.max(np.abs(U.T @ U - np.eye(d))) < 1e-12
    X = rng.standard_normal((9, d))
    Y = ho.apply(X, d, radices, blocks, sg, U=U)
    np.testing.assert_allclose(np.linalg.norm(Y, axis=1), np.linalg.norm(X, axis=1), rtol=1e-12)
    Xb = ho.apply_transpose(Y, d, radices, blocks, sg, U=U)
    assert np.max(np.abs(Xb - X)) < 1e-12


# ------------------------------------------------------------------ brute force via Eq. (7)
@pytest.mark.parametrize("radices", SCHEDULES + [[3, 4], [2, 5, 4], [7, 8], [2, 2, 2, 5], [6, 4]])
def test_bruteforce_explicit_stage_matrices(radices):
    """U from pushing the identity == diag(sigma) S_0 ... S_{m-1} with each S_t built from
    Eq. (7) as explicit permutation and block-diagonal matrices (general, non-orthogonal,
    non-symmetric blocks, so order, orientation and numbering all matter)."""
    d = int(np.prod(radices))
    blocks = _rand_blocks(d, radices, seed=100 + d, orth=False)
    sg = gi.make_signs(d, np.random.default_rng(d + 1))
    U1 = ho.build_U(d, radices, blocks, sg)
    U2 = ho.U_explicit(d, radices, blocks, sg)
    scale = np.max(np.abs(U2))
    assert np.max(np.abs(U1 - U2)) < 1e-13 * max(1.0, scale)


def test_stage_order_matters_and_is_stage0_first():
    """Apply to e_0 with stage 0 = swap inside contiguous pairs and stage 1 = a scaling that
    depends on the position: only 'stage 0 first' sends e_0 to 3*e_1."""
    d, radices = 4, [2, 2]
    swap = np.array([[0.0, 1.0], [1.0, 0.0]])
    K0 = np.stack([swap, swap])
    # stage 1 (stride 2): block beta scales by (2 + beta)
    K1 = np.stack([np.eye(2) * 2.0, np.eye(2) * 3.0])
    y = ho.apply(np.eye(d)[:1], d, radices, [K0, K1])
    np.testing.assert_array_equal(y, [[0.0, 3.0, 0.0, 0.0]])


def test_signs_act_on_input_coordinates():
    d, radices = 8, [2, 4]
    blocks = _rand_blocks(d, radices, 5, orth=False)
    sg = np.array([1, -1, 1, 1, -1, -1, 1, -1], dtype=np.int8)
    U0 = ho.build_U(d, radices, blocks)
    U = ho.build_U(d, radices, blocks, sg)
    np.testing.assert_allclose(U, np.diag(sg.astype(float)) @ U0, atol=0)


# ------------------------------------------------------------------ staged == dense, transpose
@pytest.mark.parametrize("radices", [[2] * 8, [8, 8, 4], [2, 2, 2, 2, 7], [4, 43], [3, 5, 2, 2]])
def test_staged_rows_equal_dense_definition(radices):
    d = int(np.prod(radices))
    blocks = _rand_blocks(d, radices, 11 + d, orth=True)
    sg = gi.make_signs(d, np.random.default_rng(2))
    X = np.random.default_rng(1).standard_normal((7, d))
    U = ho.build_U(d, radices, blocks, sg)
    np.testing.assert_allclose(ho.apply_staged(X, d, radices, blocks, sg), X @ U, atol=1e-12)
    np.testing.assert_allclose(ho.apply_transpose_staged(X, d, radices, blocks, sg), X @ U.T,
                               atol=1e-12)


def test_transpose_is_matrix_transpose_nonorthogonal_blocks():
    """With non-orthogonal blocks the transpose path is the matrix transpose, not the inverse."""
    d, radices = 24, [2, 3, 4]
    blocks = _rand_blocks(d, radices, 3, orth=False)
    sg = gi.make_signs(d, np.random.default_rng(4))
    U = ho.U_explicit(d, radices, blocks, sg)
    X = np.random.default_rng(5).standard_normal((4, d))
    np.testing.assert_allclose(ho.apply_transpose_staged(X, d, radices, blocks, sg), X @ U.T,
                               atol=1e-12 * np.max(np.abs(U)) * 10)


# ------------------------------------------------------------------ Kronecker identity, Eq. (12)
def test_kronecker_fallback_identity():
    """Schedule (2,2,2,K) with every last-stage block = G and pow2-stage blocks independent of
    the high digit equals G kron T_{n2} in the index order i = k*n2 + j."""
    K_, n2 = 3, 8
    d = K_ * n2
    radices = [2, 2, 2, K_]
    rng = np.random.default_rng(9)
    small = gi.make_blocks(n2, [2, 2, 2], "qr", rng)
    T_small = ho.build_U(n2, [2, 2, 2], small)
    G = gi.qr_blocks(1, K_, rng)[0].astype(np.float64)
    # tie the pow2 blocks across the K axis: block index c = alpha*s + beta, alpha = k*g_small + a
    blocks = [np.concatenate([small[t]] * K_, axis=0) for t in range(3)]
    blocks.append(np.broadcast_to(G, (n2, K_, K_)).copy())
    U = ho.build_U(d, radices, blocks)
    np.testing.assert_allclose(U, np.kron(G, T_small), atol=1e-13)


# ------------------------------------------------------------------ two-sided rotation
def test_rotate_weight_dense_and_invariance():
    do, di = 24, 40
    ru, rv = [2, 3, 4], [8, 5]
    rng = np.random.default_rng(21)
    bu = [np.linalg.qr(rng.standard_normal((do // b, b, b)))[0] for b in ru]
    bv = [np.linalg.qr(rng.standard_normal((di // b, b, b)))[0] for b in rv]
    su, sv = gi.make_signs(do, rng), gi.make_signs(di, rng)
    W = rng.standard_normal((do, di))
    Uu, Uv = ho.U_explicit(do, ru, bu, su), ho.U_explicit(di, rv, bv, sv)
    Wt = ho.rotate_weight(W, (do, ru, bu, su), (di, rv, bv, sv))
    np.testing.assert_allclose(Wt, Uu.T @ W @ Uv, atol=1e-13)
    np.testing.assert_allclose(np.linalg.norm(Wt), np.linalg.norm(W), rtol=1e-13)
    # round trip  W = U W~ V^T
    np.testing.assert_allclose(Uu @ Wt @ Uv.T, W, atol=1e-12)
    # Eq. (3): Tr((W-What) H (W-What)^T) is basis independent for any What~ and SPD H
    A = rng.standard_normal((di, di))
    H = A @ A.T + np.eye(di)
    Ht = Uv.T @ H @ Uv
    What_t = Wt + 0.1 * rng.standard_normal(Wt.shape)
    What = Uu @ What_t @ Uv.T
    lhs = np.trace((W - What) @ H @ (W - What).T)
    rhs = np.trace((Wt - What_t) @ Ht @ (Wt - What_t).T)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12)
    # one-sided variants
    np.testing.assert_allclose(ho.rotate_weight(W, None, (di, rv, bv, sv)), W @ Uv, atol=1e-13)
    np.testing.assert_allclose(ho.rotate_weight(W, (do, ru, bu, su), None), Uu.T @ W, atol=1e-13)


# ------------------------------------------------------------------ schedule helper, counts
def test_greedy_schedule_printed_examples():
    for k, v in _read_golden("greedy_schedule.txt"):
        assert ho.greedy_schedule(int(k)) == [int(x) for x in v.split()]


def test_greedy_schedule_radix_ablation_stage_counts():
    for k, v in _read_golden("radix_ablation_stage_counts.txt"):
        b = int(k)
        sched = ho.greedy_schedule(4096, b_base=b, b_max=b)
        assert len(sched) == int(v) and int(np.prod(sched)) == 4096


@pytest.mark.parametrize("d", [2, 3, 6, 43, 172, 5120, 11008, 12288, 14336, 28672, 8192, 13824])
def test_greedy_schedule_is_a_valid_schedule(d):
    sched = ho.greedy_schedule(d)
    ho.check_schedule(d, sched)


def test_param_count_literal_values():
    """Eq. (13), stage t holds d / b_t blocks with b_t (b_t - 1) / 2 free parameters each.  Values
    worked out by hand: 4096 = 8^4 -> 4 stages x 512 blocks x 28 = 57 344; 5120 = (8,8,8,5,2) ->
    3 x 640 x 28 + 1024 x 10 + 2560 x 1 = 66 560; (2,3) on d = 6 -> 3 x 1 + 2 x 3 = 9;
    11008 = 2^8 * 43 -> 8 x 5504 + 256 x 903 = 275 200."""
    assert ho.param_count(4096, [8] * 4) == 57344
    assert ho.param_count(5120, [8, 8, 8, 5, 2]) == 66560
    assert ho.param_count(6, [2, 3]) == 9
    assert ho.param_count(4, [2, 2]) == 4
    assert ho.param_count(11008, [2] * 8 + [43]) == 275200
    # and it is the number of rotation parameters the theta front end actually consumes
    d, radices = 120, [2, 3, 4, 5]
    thetas = [np.zeros((d // b, b * (b - 1) // 2)) for b in radices]
    ho.blocks_from_theta(d, radices, thetas, mixers=[np.eye(b) for b in radices])
    assert ho.param_count(d, radices) == sum(t.size for t in thetas)


# ------------------------------------------------------------------ parameterisations
def test_givens_and_cayley_special_cases():
    np.testing.assert_array_equal(ho.givens_block(0.0), np.eye(2))
    G = ho.givens_block(np.pi / 2)
    np.testing.assert_allclose(G, [[0, -1], [1, 0]], atol=1e-15)     # Eq. (10) sign convention
    for b in (3, 5, 8):
        np.testing.assert_array_equal(ho.cayley_block(np.zeros(b * (b - 1) // 2), b), np.eye(b))
        a = np.random.default_rng(b).standard_normal(b * (b - 1) // 2)
        Q = ho.cayley_block(a, b)
        np.testing.assert_allclose(Q.T @ Q, np.eye(b), atol=1e-12)
        assert np.linalg.det(Q) > 0                                   # SO(b)
    # b = 2: (I+A)^{-1}(I-A) with A = [[0,a],[-a,0]] is [[1-a^2,-2a],[2a,1-a^2]]/(1+a^2),
    # the Eq. (10) rotation by 2 atan(a)
    a = 0.37
    Q = ho.cayley_block([a], 2)
    np.testing.assert_allclose(Q, np.array([[1 - a * a, -2 * a], [2 * a, 1 - a * a]]) / (1 + a * a),
                               atol=1e-15)
    np.testing.assert_allclose(Q, ho.givens_block(2 * np.arctan(a)), atol=1e-14)


def test_cayley_radix3_is_the_rodrigues_rotation():
    """(I+A)^{-1}(I-A) with A the cross-product matrix of w is the rotation about w by
    -2 atan|w| (textbook closed form), which fixes the sign and the order of the triangle."""
    a01, a02, a12 = 0.3, -0.45, 0.8
    Q = ho.cayley_block([a01, a02, a12], 3)
    w = np.array([-a12, a02, -a01])            # A = [w]_x
    nw = np.linalg.norm(w)
    K = np.array([[0, -w[2], w[1]], [w[2], 0, -w[0]], [-w[1], w[0], 0]]) / nw
    phi = -2 * np.arctan(nw)
    R = np.eye(3) + np.sin(phi) * K + (1 - np.cos(phi)) * (K @ K)
    np.testing.assert_allclose(Q, R, atol=1e-14)
    np.testing.assert_allclose(Q @ w, w, atol=1e-14)          # the axis is fixed


@pytest.mark.parametrize("radices", [[2] * 6, [8, 8, 4], [4, 2, 8], [16, 4]])
def test_blocks_from_theta_zero_is_the_hadamard_processor(radices):
    """Theta = 0 with Hadamard mixers: every block is H_b and U = diag(sigma) H_d / sqrt(d)."""
    from scipy.linalg import hadamard
    d = int(np.prod(radices))
    blocks = ho.blocks_from_theta(d, radices, None)
    for b, K in zip(radices, blocks):
        assert K.shape == (d // b, b, b)
        np.testing.assert_allclose(K, np.broadcast_to(hadamard(b) / np.sqrt(b), K.shape), atol=1e-15)
    sig = gi.make_signs(d, np.random.default_rng(7))
    U = ho.build_U(d, radices, blocks, sig)
    np.testing.assert_allclose(U, sig[:, None] * hadamard(d) / np.sqrt(d), atol=1e-13)


def test_blocks_from_theta_forms_and_orthogonality():
    rng = np.random.default_rng(3)
    d, radices = 120, [2, 4, 3, 5]
    G3 = np.linalg.qr(rng.standard_normal((3, 3)))[0]
    thetas = [rng.standard_normal((d // b, b * (b - 1) // 2)) for b in radices]
    blocks = ho.blocks_from_theta(d, radices, thetas, [None, None, G3, "identity"])
    # radix 2: Q(theta) H_2 written out
    th = thetas[0][:, 0]
    c, s_ = np.cos(th), np.sin(th)
    want = np.stack([np.stack([c - s_, c + s_], -1), np.stack([s_ + c, s_ - c], -1)], -2) / np.sqrt(2)
    np.testing.assert_allclose(blocks[0], want, atol=1e-15)
    # radix 3 with a custom mixer, radix 5 with the identity mixer
    np.testing.assert_allclose(blocks[2][5], ho.cayley_block(thetas[2][5], 3) @ G3, atol=1e-15)
    np.testing.assert_allclose(blocks[3][2], ho.cayley_block(thetas[3][2], 5), atol=1e-15)
    for K in blocks:
        np.testing.assert_allclose(np.einsum("cij,cik->cjk", K, K), np.broadcast_to(np.eye(K.shape[1]), K.shape),
                                   atol=1e-12)
    with pytest.raises(ValueError):
        ho.blocks_from_theta(6, [2, 3], None)            # no default mixer for radix 3


# ------------------------------------------------------------------ input generator sanity
def test_bf16_rounding_is_rne_and_exact():
    x = np.array([1.0, 1.00390625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.5, 3.1415926], np.float32)
    r = gi.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0                  # tie at 1 + 2^-8 ... below: rounds down
    assert r[2] == 1.0                                  # exact tie -> even mantissa (1.0)
    assert r[3] == np.float32(1.0 + 2 ** -6)            # tie -> even (1 + 4*2^-8)
    import torch
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(r, t)
    bits = gi.bf16_bits(r)
    np.testing.assert_array_equal(gi.bf16_bits_to_f32(bits), r)


def test_generated_blocks_are_orthogonal():
    rng = np.random.default_rng(0)
    for b in (2, 3, 7, 8, 43):
        K = gi.make_blocks(b * 6, [b], "orth", rng)[0].astype(np.float64)
        err = np.max(np.abs(np.einsum("cij,cik->cjk", K, K) - np.eye(b)))
        assert err < 5e-7


# ------------------------------------------------------------------ int8 storage of Theta
def test_int8_theta_hand_computed_block():
    """App. "Int8 storage of HARP parameters": s = max|a| / 127, q = round(a / s).  One radix-3
    block (3 parameters) and radix-2 blocks (one angle each), worked by hand."""
    a3 = np.array([[0.3, -1.0, 0.26],                             # s = 1/127: 38.1, -127, 33.02
                   [2.54, 0.048, -1.0]], dtype=np.float32)        # s = 0.02: 127, 2.4, -50
    a2 = np.array([[0.5], [-2.0], [0.0]], dtype=np.float32)       # single angle -> +-127, s = |a|/127
    codes, scales = ho.quantize_theta_int8(6, [3, 2], [a3, a2])
    np.testing.assert_array_equal(codes[0], [[38, -127, 33], [127, 2, -50]])
    assert abs(float(scales[0][1]) - 0.02) < 1e-8
    assert abs(float(scales[0][0]) - 1.0 / 127.0) < 1e-9
    np.testing.assert_array_equal(codes[1], [[127], [-127], [0]])
    np.testing.assert_allclose(scales[1], [0.5 / 127, 2.0 / 127, 0.0], rtol=1e-7)
    back = ho.dequantize_theta_int8(6, [3, 2], codes, scales)
    np.testing.assert_allclose(back[0], [[38 / 127, -1.0, 33 / 127], [2.54, 0.04, -1.0]], rtol=1e-6)
    np.testing.assert_allclose(back[1], [[0.5], [-2.0], [0.0]], rtol=1e-6)


def test_int8_theta_error_bound_extremes_and_symmetry():
    rng = np.random.default_rng(5)
    d, radices = 960, [8, 5, 2, 4, 3]
    thetas = [(rng.standard_normal((d // b, b * (b - 1) // 2)) * rng.uniform(1e-3, 3.0, (d // b, 1)))
              .astype(np.float32) for b in radices]
    codes, scales = ho.quantize_theta_int8(d, radices, thetas)
    back = ho.dequantize_theta_int8(d, radices, codes, scales)
    neg_codes, neg_scales = ho.quantize_theta_int8(d, radices, [-t for t in thetas])
    for t, b in enumerate(radices):
        assert codes[t].dtype == np.int8 and scales[t].dtype == np.float32
        assert codes[t].min() >= -127
        # the largest parameter of every block sits at +-127
        assert np.all(np.max(np.abs(codes[t].astype(np.int32)), axis=1) == 127)
        # rounding error at most half a step (plus float32 rounding of the quotient and product)
        err = np.abs(back[t].astype(np.float64) - thetas[t].astype(np.float64))
        assert np.all(err <= 0.5 * scales[t][:, None].astype(np.float64) * (1 + 1e-5))
        # odd symmetry of round-half-even
        np.testing.assert_array_equal(neg_codes[t], -codes[t])
        np.testing.assert_array_equal(neg_scales[t], scales[t])
    # the reconstructed blocks are orthogonal and close to the unquantised ones
    Kq = ho.blocks_from_theta(d, radices, back, ["hadamard", "identity", None, None, "identity"])
    K = ho.blocks_from_theta(d, radices, thetas, ["hadamard", "identity", None, None, "identity"])
    for kq, k in zip(Kq, K):
        eye = np.einsum("cij,ckj->cik", kq, kq)
        assert np.max(np.abs(eye - np.eye(kq.shape[1]))) < 1e-12
        assert np.max(np.abs(kq - k)) < 0.2


# ------------------------------------------------------------------ gradient through the stages
def _loss(X, G, d, radices, blocks, signs):
    return float(np.sum(ho.apply(X, d, radices, blocks, signs) * G))


@pytest.mark.parametrize("d,radices", [(12, [2, 3, 2]), (16, [4, 2, 2]), (30, [5, 2, 3])])
def test_grad_blocks_against_central_finite_differences(d, radices):
    """L = <apply(X), G> is linear in every block entry, so a central difference is exact up to
    rounding: every entry of every dK, and every entry of dX, is checked."""
    rng = np.random.default_rng(d)
    blocks = [rng.standard_normal((d // b, b, b)) for b in radices]       # not orthogonal on purpose
    signs = rng.choice([-1, 1], size=d).astype(np.int8)
    X, G = rng.standard_normal((5, d)), rng.standard_normal((5, d))
    dK, dX = ho.grad_blocks(X, G, d, radices, blocks, signs)
    h = 1e-3
    for t, b in enumerate(radices):
        for c in range(d // b):
            for r in range(b):
                for r2 in range(b):
                    bp = [k.copy() for k in blocks]
                    bm = [k.copy() for k in blocks]
                    bp[t][c, r, r2] += h
                    bm[t][c, r, r2] -= h
                    fd = (_loss(X, G, d, radices, bp, signs) - _loss(X, G, d, radices, bm, signs)) / (2 * h)
                    assert abs(fd - dK[t][c, r, r2]) < 1e-8 * (1 + abs(fd)), (t, c, r, r2)
    for i in range(X.shape[0]):
        for j in range(d):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, j] += h
            Xm[i, j] -= h
            fd = (_loss(Xp, G, d, radices, blocks, signs) - _loss(Xm, G, d, radices, blocks, signs)) / (2 * h)
            assert abs(fd - dX[i, j]) < 1e-8 * (1 + abs(fd))


def test_grad_blocks_closed_forms_and_linearity():
    rng = np.random.default_rng(3)
    d, radices = 48, [4, 3, 2, 2]
    blocks = gi.make_blocks(d, radices, "orth", rng)
    signs = gi.make_signs(d, rng)
    X, G = rng.standard_normal((9, d)), rng.standard_normal((9, d))
    dK, dX = ho.grad_blocks(X, G, d, radices, blocks, signs)
    # dX = G U^T through the dense matrix
    U = ho.build_U(d, radices, blocks, signs)
    np.testing.assert_allclose(dX, G @ U.T, atol=1e-12)
    # a single stage (b = d, one block): dK = (X * sigma)^T G
    d1 = 6
    K1 = [rng.standard_normal((1, d1, d1))]
    s1 = rng.choice([-1, 1], size=d1).astype(np.int8)
    X1, G1 = rng.standard_normal((7, d1)), rng.standard_normal((7, d1))
    dK1, dX1 = ho.grad_blocks(X1, G1, d1, [d1], K1, s1)
    np.testing.assert_allclose(dK1[0][0], (X1 * s1).T @ G1, atol=1e-12)
    np.testing.assert_allclose(dX1, (G1 @ K1[0][0].T) * s1, atol=1e-12)
    # the last stage of a longer schedule: its input is the transform by the earlier stages
    xin = X * signs
    stv = ho.strides(radices)
    for t in range(len(radices) - 1):
        xin = ho.stage_apply_rows(xin.copy(), radices[t], stv[t], np.asarray(blocks[t], dtype=np.float64))
    bl, sl = radices[-1], stv[-1]
    for c in (0, d // bl - 1):
        idx = (c // sl) * bl * sl + np.arange(bl) * sl + c % sl
        np.testing.assert_allclose(dK[-1][c], xin[:, idx].T @ G[:, idx], atol=1e-12)
    # linear in G, and rows add up
    dK2, _ = ho.grad_blocks(X, 2.0 * G, d, radices, blocks, signs)
    dKa, _ = ho.grad_blocks(X[:4], G[:4], d, radices, blocks, signs)
    dKb, _ = ho.grad_blocks(X[4:], G[4:], d, radices, blocks, signs)
    for t in range(len(radices)):
        np.testing.assert_allclose(dK2[t], 2.0 * dK[t], atol=1e-12)
        np.testing.assert_allclose(dKa[t] + dKb[t], dK[t], atol=1e-12)
