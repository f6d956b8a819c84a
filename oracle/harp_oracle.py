"""CPU float64 oracle for the HARP structured-rotation path.  TEST INFRASTRUCTURE ONLY.

This module is the checker, not the product: only ``tests/``, the smoke entry and
the ``cpu_baseline`` leg of the benchmark may import it.  It shares no code with
the HIP library and never imports it.

What it computes (paper Sec. 3, Eq. (6)-(8), Alg. 1; App. A Lemma 1; Sec. 2 for
the two-sided change of basis):

* a HARP processor is a Mixed-Radix schedule ``b = (b_0..b_{m-1})`` with
  ``prod b_t = d``, one dense ``b_t x b_t`` block per stride group and stage, and a
  +-1 sign vector;
* stage ``t`` has stride ``s_t = prod_{j<t} b_j`` and ``g_t = d / (b_t s_t)`` groups;
  for every ``(alpha, beta)``, ``alpha < g_t``, ``beta < s_t`` it takes the ``b_t``
  coordinates ``alpha*b_t*s_t + r*s_t + beta`` (Lemma 1's flattening), multiplies that
  row vector by block ``c = alpha*s_t + beta`` on the right and puts the result back;
* the transform runs stage 0 first (Alg. 1's loop order);
* ``apply(x) = T(x * sigma)`` so ``U = diag(sigma) T``; ``apply_transpose(x) = x U^T``;
* ``rotate_weight(W) = U_U^T W U_V``.

HARP is an exact factorisation, so the reference result has a plain definition:
materialise ``U`` as a dense float64 matrix by pushing the signed identity through
the stages and form ``X @ U``.  That is ``build_U`` / ``apply`` below.  ``apply_staged``
is Alg. 1 taken step by step on the rows themselves (no dense ``U``); it exists so
that rows of very long transforms (d > 8192) can be checked one by one, and it is
pinned against the dense definition in the CPU tests.  ``stage_matrix_explicit`` is a
third, independent formulation (Eq. (7): permutation * block-diagonal * permutation^T)
used only to pin the other two at small d.

Readings of the paper where it is silent (each also listed in the design notes):
row vector on the left of the block (``v' = v K``), block numbering
``c = alpha*s_t + beta``, signs on the input coordinates of ``apply``.

Pins (tests/test_oracle_*.py): Lemma 1 index example (d=16, b=4), Kronecker closed
form of a stage, Theta=0 power-of-two schedules equal the normalised Sylvester
Hadamard (checked against scipy's hadamard), U^T U = I, norm preservation, round
trip, brute force through Eq. (7) at d <= 172, transpose equals matrix transpose,
loss invariance Eq. (3), the greedy schedule's printed examples (App. "Stage
schedules", Alg. 2) and Table "radix ablation" stage counts, Eq. (13) parameter count;
``blocks_from_theta``: Theta = 0 gives diag(sigma) H_d / sqrt(d) (scipy's hadamard), the
radix-2 block written out, the radix-3 Cayley block against the Rodrigues rotation.
``quantize_theta_int8`` (App. "Int8 storage of HARP parameters"): a hand-computed block, the
largest parameter of a block mapping to +-127, |a - s q| <= s / 2, sign symmetry.
``grad_blocks`` (the gradient that Alg. 3's update needs, by the chain rule through Alg. 1):
central finite differences of <apply(X), G> in every block entry at small d, dX = G U^T
through the dense U, the single-stage closed form X_sigma[:, idx]^T G[:, idx], linearity in G.
Unpinned against the paper (values not published): the QR base mixer's fixed
Gaussian and any trained processor -- "parity unpinned" for those; they are inputs
to this library, not computed by it.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "check_schedule", "strides", "stage_apply_rows", "transform_rows",
    "transform_rows_transpose", "build_U", "apply", "apply_transpose",
    "apply_staged", "apply_transpose_staged", "rotate_weight",
    "stage_matrix_explicit", "U_explicit", "greedy_schedule",
    "sylvester_hadamard", "param_count", "givens_block", "cayley_block",
    "blocks_from_theta", "quantize_theta_int8", "dequantize_theta_int8", "grad_blocks",
]


# --------------------------------------------------------------------------- schedule
def check_schedule(d, radices):
    """Eq. (6): every radix >= 2 and their product equals d."""
    radices = [int(b) for b in radices]
    if d < 1 or len(radices) == 0:
        raise ValueError("empty schedule or non-positive d")
    if any(b < 2 for b in radices):
        raise ValueError("every radix must be >= 2")
    p = 1
    for b in radices:
        p *= b
    if p != d:
        raise ValueError(f"product of radices {p} != d {d}")
    return radices


def strides(radices):
    """s_0 = 1, s_t = prod_{j<t} b_j  (Sec. 3 after Eq. (6); Alg. 1 'precompute strides')."""
    s, out = 1, []
    for b in radices:
        out.append(s)
        s *= int(b)
    return out


def _as_blocks(d, radices, blocks):
    """Widen the caller's blocks to float64 exactly; shape-check [D_t, b_t, b_t]."""
    out = []
    for t, b in enumerate(radices):
        K = np.asarray(blocks[t], dtype=np.float64)
        if K.shape != (d // b, b, b):
            raise ValueError(f"stage {t}: blocks shape {K.shape} != {(d // b, b, b)}")
        out.append(K)
    return out


def _as_signs(d, signs):
    if signs is None:
        return np.ones(d, dtype=np.float64)
    s = np.asarray(signs, dtype=np.float64)
    if s.shape != (d,) or not np.all(np.abs(s) == 1.0):
        raise ValueError("signs must be d values in {+1,-1}")
    return s


# --------------------------------------------------------------------------- one stage
def stage_apply_rows(Y, b, s, K, transpose_blocks=False):
    """One stage of Alg. 1 on every row of Y (in place), Lemma 1 indexing.

    For each group index alpha and within-stride offset beta, the b coordinates
    ``alpha*b*s + r*s + beta`` (r = 0..b-1) form a row vector v; it is replaced by
    ``v @ K[c]`` with ``c = alpha*s + beta`` (or ``v @ K[c].T`` for the transposed stage).
    """
    n, d = Y.shape
    g = d // (b * s)
    r = np.arange(b)
    for alpha in range(g):
        for beta in range(s):
            c = alpha * s + beta
            idx = alpha * b * s + r * s + beta
            M = K[c].T if transpose_blocks else K[c]
            Y[:, idx] = Y[:, idx] @ M
    return Y


def transform_rows(Y, radices, blocks):
    """y <- T(y) on every row: stages t = 0, 1, ..., m-1 in that order (Alg. 1 loop)."""
    st = strides(radices)
    for t, b in enumerate(radices):
        stage_apply_rows(Y, b, st[t], blocks[t])
    return Y


def transform_rows_transpose(Y, radices, blocks):
    """y <- y T^T: the stages in reverse order, each block transposed."""
    st = strides(radices)
    for t in range(len(radices) - 1, -1, -1):
        stage_apply_rows(Y, radices[t], st[t], blocks[t], transpose_blocks=True)
    return Y


# --------------------------------------------------------------------------- dense U
def build_U(d, radices, blocks, signs=None):
    """Dense float64 U with apply(x) = x @ U: row i of U is T(sigma_i e_i)."""
    radices = check_schedule(d, radices)
    K = _as_blocks(d, radices, blocks)
    sg = _as_signs(d, signs)
    Y = np.diag(sg)                      # signed identity, one basis vector per row
    return transform_rows(Y, radices, K)


def apply(X, d, radices, blocks, signs=None, U=None):
    """Y = X U (the definition).  X is widened to float64 exactly; result unrounded."""
    if U is None:
        U = build_U(d, radices, blocks, signs)
    return np.asarray(X, dtype=np.float64) @ U


def apply_transpose(X, d, radices, blocks, signs=None, U=None):
    """Y = X U^T."""
    if U is None:
        U = build_U(d, radices, blocks, signs)
    return np.asarray(X, dtype=np.float64) @ U.T


def rotate_weight(W, plan_U=None, plan_V=None):
    """W~ = U_U^T W U_V (Sec. 2, two-sided change of basis).

    plan_* = (d, radices, blocks, signs) or None for the identity on that side.
    """
    W = np.asarray(W, dtype=np.float64)
    out = W
    if plan_V is not None:
        out = out @ build_U(*plan_V)
    if plan_U is not None:
        out = build_U(*plan_U).T @ out
    return out


# --------------------------------------------------------------------------- staged rows
def apply_staged(X, d, radices, blocks, signs=None):
    """Alg. 1 on the rows themselves: T(x * sigma).  Equals ``apply`` (pinned in tests)."""
    radices = check_schedule(d, radices)
    K = _as_blocks(d, radices, blocks)
    sg = _as_signs(d, signs)
    Y = np.array(X, dtype=np.float64) * sg[None, :]
    return transform_rows(Y, radices, K)


def apply_transpose_staged(X, d, radices, blocks, signs=None):
    """(x T^T) * sigma on every row.  Equals ``apply_transpose`` (pinned in tests)."""
    radices = check_schedule(d, radices)
    K = _as_blocks(d, radices, blocks)
    sg = _as_signs(d, signs)
    Y = np.array(X, dtype=np.float64)
    transform_rows_transpose(Y, radices, K)
    return Y * sg[None, :]


# --------------------------------------------------------------------------- Eq. (7) form
def stage_matrix_explicit(d, b, s, K):
    """Row-convention stage matrix via Eq. (7): Pi * BlkDiag(K_0..K_{D-1}) * Pi^T.

    pi(alpha*b*s + r*s + beta) = (alpha*s + beta)*b + r is the perfect shuffle that makes
    each stride group contiguous; Pi[i, pi(i)] = 1.  y = x @ (Pi B Pi^T).  Built
    element by element with scalar loops, no use of the routines above.
    """
    K = np.asarray(K, dtype=np.float64)
    D = d // b
    Pi = np.zeros((d, d))
    g = d // (b * s)
    for alpha in range(g):
        for r in range(b):
            for beta in range(s):
                Pi[alpha * b * s + r * s + beta, (alpha * s + beta) * b + r] = 1.0
    B = np.zeros((d, d))
    for c in range(D):
        B[c * b:(c + 1) * b, c * b:(c + 1) * b] = K[c]
    return Pi @ B @ Pi.T


def U_explicit(d, radices, blocks, signs=None):
    """diag(sigma) S_0 S_1 ... S_{m-1} with every factor an explicit dense matrix."""
    radices = check_schedule(d, radices)
    st = strides(radices)
    U = np.diag(_as_signs(d, signs))
    for t, b in enumerate(radices):
        U = U @ stage_matrix_explicit(d, b, st[t], blocks[t])
    return U


# --------------------------------------------------------------------------- helpers
def greedy_schedule(d, b_base=8, b_max=8):
    """Greedy Mixed-Radix schedule (Alg. 2): peel the preferred radix while it divides,
    then factors from min(b_max, r) down to 2, then any leftover as a last stage."""
    if d < 2:
        raise ValueError("d must be >= 2")
    out, r = [], int(d)
    while r % b_base == 0:
        out.append(b_base)
        r //= b_base
    for f in range(min(b_max, r), 1, -1):
        while r % f == 0:
            out.append(f)
            r //= f
    if r != 1:
        out.append(r)
    return out


def sylvester_hadamard(b):
    """Normalised Sylvester Hadamard H_b = b^{-1/2} H~_b, H~_{2n} = [[H,H],[H,-H]] (App. A)."""
    if b < 1 or (b & (b - 1)) != 0:
        raise ValueError("b must be a power of two")
    H = np.ones((1, 1))
    while H.shape[0] < b:
        H = np.block([[H, H], [H, -H]])
    return H / np.sqrt(b)


def param_count(d, radices):
    """Eq. (13): sum_t D_t b_t (b_t - 1) / 2 = sum_t d (b_t - 1) / 2."""
    return sum((d // b) * (b * (b - 1) // 2) for b in radices)


def givens_block(theta):
    """Eq. (10), as printed: [[cos, -sin], [sin, cos]]."""
    c, s = np.cos(theta), np.sin(theta)
    return np.array([[c, -s], [s, c]])


def cayley_block(upper, b):
    """Eq. (11): Q = (I + A)^{-1} (I - A), A skew-symmetric with the given strict upper
    triangle (row-major order (0,1), (0,2), ...)."""
    A = np.zeros((b, b))
    iu = np.triu_indices(b, 1)
    A[iu] = np.asarray(upper, dtype=np.float64)
    A = A - A.T
    I = np.eye(b)
    return np.linalg.solve(I + A, I - A)


def blocks_from_theta(d, radices, thetas, mixers=None):
    """Block kernels B_{t,c} = Q(theta_{t,c}) G_{b_t} (Eq. (9)), as float64 arrays [D_t, b_t, b_t].

    thetas[t]: None (all zeros: Q = I, Sec. 3 'Exact initialization'), or an array
    [D_t, b_t (b_t - 1) / 2]: the rotation angle for b_t = 2 (Eq. (10)), the strict upper
    triangle of the skew-symmetric A for b_t > 2 (Eq. (11)).  mixers[t]: None = the normalised
    Sylvester Hadamard matrix (power-of-two radices only; also the string "hadamard"), the
    string "identity", or an
    explicit orthogonal b_t x b_t matrix (the paper's QR fallback for other radices is a seeded
    matrix whose seed is not published, so it has to be supplied).  The product is taken as
    printed, Q then G, and the block is used as v -> v B like any other block.
    """
    check_schedule(d, radices)
    out = []
    for t, b in enumerate(radices):
        D = d // b
        G = None if mixers is None else mixers[t]
        if G is None or (isinstance(G, str) and G == "hadamard"):
            if b & (b - 1):
                raise ValueError("no default base mixer for a radix that is not a power of two")
            G = sylvester_hadamard(b)
        elif isinstance(G, str):
            if G != "identity":
                raise ValueError("unknown mixer")
            G = np.eye(b)
        else:
            G = np.asarray(G, dtype=np.float64)
            if G.shape != (b, b):
                raise ValueError("mixer shape")
        npar = b * (b - 1) // 2
        th = None if thetas is None or thetas[t] is None else np.asarray(thetas[t], dtype=np.float64).reshape(D, npar)
        K = np.empty((D, b, b))
        for c in range(D):
            if th is None:
                Q = np.eye(b)
            elif b == 2:
                Q = givens_block(th[c, 0])
            else:
                Q = cayley_block(th[c], b)
            K[c] = Q @ G
        out.append(K)
    return out



def quantize_theta_int8(d, radices, thetas):
    """Int8 storage of the stage parameters (App. "Int8 storage of HARP parameters").

    For block c of stage t with parameters a (the strict upper triangle of A for b_t > 2, the
    Givens angle for b_t = 2):  s = max|a| / 127,  q = round(a / s).  The paper fixes neither the
    precision nor the tie rule; both are taken as float32 and round-half-to-even (what the
    float32 tensor code the paper describes would do), and a block of zeros gets s = 0, q = 0.
    Returns (codes, scales): int8 arrays [D_t, p_t] and float32 arrays [D_t].
    """
    check_schedule(d, radices)
    codes, scales = [], []
    for t, b in enumerate(radices):
        D, npar = d // b, b * (b - 1) // 2
        a = np.asarray(thetas[t], dtype=np.float32).reshape(D, npar)
        q = np.zeros((D, npar), dtype=np.int8)
        s = np.zeros(D, dtype=np.float32)
        for c in range(D):
            amax = np.float32(np.max(np.abs(a[c])))
            s[c] = amax / np.float32(127.0)
            if s[c] > 0:
                for i in range(npar):
                    r = np.rint(np.float32(a[c, i]) / s[c])      # float32 quotient, ties to even
                    q[c, i] = np.int8(min(127.0, max(-127.0, float(r))))
        codes.append(q)
        scales.append(s)
    return codes, scales


def dequantize_theta_int8(d, radices, codes, scales):
    """a ~ s * q in float32 (same appendix), arrays [D_t, p_t] per stage."""
    check_schedule(d, radices)
    out = []
    for t, b in enumerate(radices):
        D, npar = d // b, b * (b - 1) // 2
        q = np.asarray(codes[t], dtype=np.int8).reshape(D, npar)
        s = np.asarray(scales[t], dtype=np.float32).reshape(D)
        out.append((s[:, None] * q.astype(np.float32)).astype(np.float32))
    return out


def grad_blocks(X, G, d, radices, blocks, signs=None):
    """Gradient of a loss through ``Y = apply(X)`` with respect to every block entry and to X,
    given ``G = dL/dY`` -- what the update of Alg. 3 (layerwise fitting) differentiates.

    Chain rule through Alg. 1, stage by stage.  Forward: ``x_0 = X * sigma``, ``x_{t+1} =
    stage_t(x_t)``.  Backward from ``g_m = G``: for block c of stage t with coordinates idx,
    ``dK_t[c] = x_t[:, idx]^T @ g_{t+1}[:, idx]`` (sum over the rows) and
    ``g_t[:, idx] = g_{t+1}[:, idx] @ K_t[c]^T``; finally ``dX = g_0 * sigma``.
    Returns (dK, dX): a list of float64 arrays [D_t, b_t, b_t], and [n, d].
    """
    radices = check_schedule(d, radices)
    K = _as_blocks(d, radices, blocks)
    sg = _as_signs(d, signs)
    st = strides(radices)
    m = len(radices)
    x = [np.array(X, dtype=np.float64) * sg[None, :]]
    for t, b in enumerate(radices):
        x.append(stage_apply_rows(x[t].copy(), b, st[t], K[t]))
    g = np.array(G, dtype=np.float64)
    if g.shape != x[0].shape:
        raise ValueError("G must have the shape of X")
    dK = [None] * m
    for t in range(m - 1, -1, -1):
        b, s = radices[t], st[t]
        D = d // b
        dKt = np.empty((D, b, b))
        r = np.arange(b)
        gn = np.empty_like(g)
        for alpha in range(d // (b * s)):
            for beta in range(s):
                c = alpha * s + beta
                idx = alpha * b * s + r * s + beta
                dKt[c] = x[t][:, idx].T @ g[:, idx]
                gn[:, idx] = g[:, idx] @ K[t][c].T
        dK[t] = dKt
        g = gn
    return dK, g * sg[None, :]
