"""Seeded synthetic inputs for the HARP rotation path (numpy only).

This module produces *inputs* -- activations, weights, per-stage block kernels, sign
vectors -- with the shapes and value character of the paper's workloads (Llama hidden
sizes 4096 / 11008 / 14336 / 28672, heavy-tailed activations with a few outlier
channels, Sec. 2 "Incoherence processing").  It applies no stage, no transform and no
rotation: both the CPU oracle's tests and the GPU harness draw from it, and nothing
else is shared between them.

Every tensor is a deterministic function of (config id, role): the generator is
``numpy.random.default_rng(1000 * config + role)`` with role 0 = X, 1 = blocks,
2 = signs, 3 = outlier channel choice, 4 = W.  Values destined for bf16 I/O are rounded
to bf16 (round to nearest even) once, here, and returned as float32 holding exactly
representable values, so both sides consume identical numbers.
"""
from __future__ import annotations

import math

import numpy as np

ROLE_X, ROLE_BLOCKS, ROLE_SIGNS, ROLE_OUTLIER, ROLE_W = 0, 1, 2, 3, 4


def rng_for(config: int, role: int) -> np.random.Generator:
    return np.random.default_rng(1000 * int(config) + int(role))


# ------------------------------------------------------------------ number formats
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bf16 (ties to even); result is float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values already exactly representable in bf16."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value not representable in bf16"
    return (u >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ------------------------------------------------------------------ schedules
def radix2_chain(d: int, last: int | None = None) -> list[int]:
    """[2]*k (+ [last]) with 2^k * last == d."""
    q = d if last is None else d // last
    k = int(round(math.log2(q)))
    assert (1 << k) * (1 if last is None else last) == d, (d, last)
    return [2] * k + ([] if last is None else [last])


def uniform_radix(d: int, b: int) -> list[int]:
    m = int(round(math.log(d, b)))
    assert b ** m == d, (d, b)
    return [b] * m


# ------------------------------------------------------------------ block kernels
def givens_blocks(D: int, rng: np.random.Generator) -> np.ndarray:
    """D rotations [[c,-s],[s,c]] with angles uniform on [0, 2 pi); float32 [D,2,2]."""
    th = rng.uniform(0.0, 2.0 * np.pi, size=D)
    c, s = np.cos(th), np.sin(th)
    K = np.empty((D, 2, 2), dtype=np.float64)
    K[:, 0, 0], K[:, 0, 1], K[:, 1, 0], K[:, 1, 1] = c, -s, s, c
    return K.astype(np.float32)


def qr_blocks(D: int, b: int, rng: np.random.Generator) -> np.ndarray:
    """D orthogonal b x b blocks: Q factor of a standard Gaussian matrix, columns
    re-signed so that R's diagonal is positive (a deterministic function of the draw)."""
    G = rng.standard_normal((D, b, b))
    Q, R = np.linalg.qr(G)
    sg = np.sign(np.diagonal(R, axis1=1, axis2=2))
    sg[sg == 0] = 1.0
    return (Q * sg[:, None, :]).astype(np.float32)


def hadamard_blocks(D: int, b: int) -> np.ndarray:
    """D copies of the normalised Sylvester Hadamard matrix of order b (b a power of 2)."""
    H = np.ones((1, 1))
    while H.shape[0] < b:
        H = np.block([[H, H], [H, -H]])
    assert H.shape[0] == b
    return np.broadcast_to((H / np.sqrt(b)).astype(np.float32), (D, b, b)).copy()


def generic_blocks(D: int, b: int, rng: np.random.Generator) -> np.ndarray:
    """D non-orthogonal, well-conditioned b x b blocks: I + (0.3 / sqrt(b)) N(0,1), so the
    perturbation has spectral norm about 0.6 whatever the radix; float32 [D,b,b]."""
    K = np.eye(b)[None, :, :] + (0.3 / math.sqrt(b)) * rng.standard_normal((D, b, b))
    return K.astype(np.float32)


BLOCK_KINDS = ("orth", "hadamard", "qr", "generic")


def make_blocks(d: int, radices, kind: str, rng: np.random.Generator):
    """Per-stage block arrays [d/b_t, b_t, b_t] float32.

    kind: 'orth' -> Givens for radix 2, sign-fixed QR otherwise;
          'hadamard' -> Theta = 0 initialisation (power-of-two radices only);
          'qr' -> sign-fixed QR for every radix (includes reflections at radix 2);
          'generic' -> non-orthogonal blocks I + (0.3 / sqrt(b)) N(0,1) at every radix."""
    if kind not in BLOCK_KINDS:
        raise ValueError(f"unknown block kind {kind!r}; one of {BLOCK_KINDS}")
    out = []
    for b in radices:
        D = d // b
        if kind == "hadamard":
            out.append(hadamard_blocks(D, b))
        elif kind == "generic":
            out.append(generic_blocks(D, b, rng))
        elif kind == "qr" or b != 2:
            out.append(qr_blocks(D, b, rng))
        else:
            out.append(givens_blocks(D, rng))
    return out


def hadamard_table(K: int) -> np.ndarray:
    """A K x K matrix with entries +-1 and H H^T = K I (float32), by Paley's constructions:
    order q + 1 for a prime q = 3 (mod 4), order 2 (q + 1) for a prime q = 1 (mod 4), doubled
    (Sylvester) as often as needed.  Covers 2, 4, 8, 12, 16, 20, 24, 28, 32, 36, 40, 44, 48, 56, 60, 64."""
    def is_prime(q):
        return q >= 2 and all(q % p for p in range(2, int(q ** 0.5) + 1))

    def jacobsthal(q):
        res = {(x * x) % q for x in range(1, q)}
        return np.array([[0 if i == j else (1 if ((i - j) % q) in res else -1) for j in range(q)]
                         for i in range(q)], dtype=np.int64)

    def build(k):
        if k == 1:
            return np.ones((1, 1), dtype=np.int64)
        if k == 2:
            return np.array([[1, 1], [1, -1]], dtype=np.int64)
        q = k - 1
        if k % 4 == 0 and is_prime(q) and q % 4 == 3:           # Paley I
            S = np.zeros((k, k), dtype=np.int64)
            S[0, 1:] = 1
            S[1:, 0] = -1
            S[1:, 1:] = jacobsthal(q)
            return np.eye(k, dtype=np.int64) + S
        q = k // 2 - 1
        if k % 4 == 0 and is_prime(q) and q % 4 == 1:           # Paley II
            C0 = np.zeros((q + 1, q + 1), dtype=np.int64)       # symmetric conference matrix
            C0[0, 1:] = 1
            C0[1:, 0] = 1
            C0[1:, 1:] = jacobsthal(q)
            A = np.array([[1, 1], [1, -1]], dtype=np.int64)
            B = np.array([[1, -1], [-1, -1]], dtype=np.int64)
            return np.kron(C0, A) + np.kron(np.eye(q + 1, dtype=np.int64), B)
        if k % 2 == 0:
            h = build(k // 2)
            return np.block([[h, h], [h, -h]])
        raise ValueError(f"no construction for a Hadamard matrix of order {k} here")

    H = build(int(K))
    assert np.array_equal(H @ H.T, K * np.eye(K, dtype=np.int64)), K
    return H.astype(np.float32)


def make_signs(d: int, rng: np.random.Generator) -> np.ndarray:
    return (rng.integers(0, 2, size=d).astype(np.int8) * 2 - 1).astype(np.int8)


# ------------------------------------------------------------------ activations / weights
def activations(n: int, d: int, config: int, dist: str = "student_t", nu: float = 3.0,
                outlier_frac: float = 0.01, outlier_scale: float = 20.0,
                bf16: bool = True) -> np.ndarray:
    """n x d float32.  dist 'normal' -> N(0,1); 'student_t' -> Student-t(nu).
    ceil(outlier_frac * d) channels, chosen with the role-3 generator, are scaled by
    outlier_scale.  bf16=True rounds once to bf16-representable values."""
    rng = rng_for(config, ROLE_X)
    if dist == "normal":
        X = rng.standard_normal((n, d))
    elif dist == "student_t":
        X = rng.standard_t(nu, size=(n, d))
    else:
        raise ValueError(dist)
    k = int(math.ceil(outlier_frac * d)) if outlier_frac > 0 else 0
    if k:
        ch = rng_for(config, ROLE_OUTLIER).choice(d, size=k, replace=False)
        X[:, ch] *= outlier_scale
    X = X.astype(np.float32)
    return round_to_bf16(X) if bf16 else X


def weights(d_out: int, d_in: int, config: int, std: float = 0.02, bf16: bool = True):
    W = (rng_for(config, ROLE_W).standard_normal((d_out, d_in)) * std).astype(np.float32)
    return round_to_bf16(W) if bf16 else W


def processor(d: int, radices, config: int, kind: str = "orth", with_signs: bool = True,
              salt: int = 0):
    """(blocks, signs) for one processor; ``salt`` separates U and V of one config."""
    blocks = make_blocks(d, radices, kind, np.random.default_rng(
        1000 * config + ROLE_BLOCKS + 100 * salt))
    signs = make_signs(d, np.random.default_rng(1000 * config + ROLE_SIGNS + 100 * salt)) \
        if with_signs else None
    return blocks, signs


# ------------------------------------------------------------------ named workloads
WORKLOADS = {
    # name: (n, d, radices, I/O dtype, activation recipe)
    "tiny_256_r2": dict(config=1, n=64, d=256, radices=[2] * 8, dtype="f32",
                        act=dict(dist="normal", outlier_frac=0.0, bf16=False)),
    "llama7b_4096_r2": dict(config=2, n=2048, d=4096, radices=[2] * 12, dtype="bf16",
                            act=dict(dist="student_t", outlier_frac=0.01, outlier_scale=20.0)),
    "llama7b_4096_r8": dict(config=2, n=2048, d=4096, radices=[8] * 4, dtype="bf16",
                            act=dict(dist="student_t", outlier_frac=0.01, outlier_scale=20.0)),
    "down_11008_r2x8_43": dict(config=3, n=2048, d=11008, radices=[2] * 8 + [43], dtype="bf16",
                               act=dict(dist="student_t", outlier_frac=0.01, outlier_scale=20.0)),
    "ffn_14336_r2x11_7": dict(config=3, n=2048, d=14336, radices=[2] * 11 + [7], dtype="bf16",
                              act=dict(dist="student_t", outlier_frac=0.01, outlier_scale=20.0)),
    # Llama-2-13B widths (hidden 5120 = 2^10 * 5, FFN 13824 = 2^9 * 27): same recipe as config 3
    "llama13b_5120_r2x10_5": dict(config=3, n=2048, d=5120, radices=[2] * 10 + [5], dtype="bf16",
                                  act=dict(dist="student_t", outlier_frac=0.01, outlier_scale=20.0)),
    "ffn13b_13824_r2x9_27": dict(config=3, n=2048, d=13824, radices=[2] * 9 + [3, 3, 3], dtype="bf16",
                                 act=dict(dist="student_t", outlier_frac=0.01, outlier_scale=20.0)),
    # hidden size of the 70B models (8192 = 2^13): same recipe as config 5's activations
    "hidden70b_8192_r2": dict(config=5, n=2048, d=8192, radices=[2] * 13, dtype="bf16",
                              act=dict(dist="student_t", outlier_frac=0.01, outlier_scale=20.0)),
    "ffn70b_28672_r2x12_7": dict(config=5, n=4096, d=28672, radices=[2] * 12 + [7], dtype="bf16",
                                 act=dict(dist="student_t", outlier_frac=0.01, outlier_scale=20.0)),
}


def workload(name: str, n: int | None = None, kind: str = "orth"):
    """Materialise a named workload: dict with X (float32), blocks, signs and metadata."""
    w = dict(WORKLOADS[name])
    if n is not None:
        w["n"] = n
    w["X"] = activations(w["n"], w["d"], w["config"], **w["act"])
    w["blocks"], w["signs"] = processor(w["d"], w["radices"], w["config"], kind=kind)
    w["name"] = name
    return w
