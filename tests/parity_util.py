"""Helpers for the GPU parity tests: tensor marshalling and the elementwise tolerance.

Tolerance (the spec bar, made precise with a row-scale floor because rotated outputs
pass through zero): with rho_i = ||Yref[i,:]||_2 / sqrt(d),
  float32 I/O :  |Y - Yref|_ij <= 1e-5 * max(|Yref_ij|, rho_i)
  bfloat16 I/O:  |Y - Yref|_ij <= ulp_bf16(Yref_ij) + 4e-3 * max(|Yref_ij|, rho_i)
where ulp_bf16(y) = 2^(floor(log2|y|) - 7) (spacing of bf16 numbers at y).

That bar is stated for orthogonal processors, whose intermediates have the size of the output.
With non-orthogonal blocks an output entry can be a small difference of large summands, so the
float32 rounding of the path is relative to the summands, not to the result: those cases pass
`mag` = the same processor applied to |X| with |blocks| (an entrywise bound on the summands of
every output, from `summand_magnitude`), and the tolerance grows by 2e-6 * mag (a chain of
m <= 30 float32 stages accumulates at most about m * 6e-8 of it).

`rho` replaces the scale floor where the processor does not act along the rows of the array
that is compared: in U^T W the vectors that plan_U transforms are the COLUMNS of W, so the
same bar read along the direction of the transform has rho_j = ||W[:,j]||_2 / sqrt(d_out) (a
column's norm is preserved by an orthogonal U, so it is known without the full result).
"""
import numpy as np

from paper_2605_29843_amd import inputs as gi


def to_device(a: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        bits = gi.bf16_bits(a)
        return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host64(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def ulp_bf16(y: np.ndarray) -> np.ndarray:
    a = np.abs(y)
    e = np.floor(np.log2(np.maximum(a, 1e-300)))
    e = np.maximum(e, -126.0)
    return np.where(a > 0, 2.0 ** (e - 7), 2.0 ** -133)


def tolerance(Yref: np.ndarray, dtype: str, rho=None) -> np.ndarray:
    d = Yref.shape[1]
    if rho is None:
        rho = np.linalg.norm(Yref, axis=1, keepdims=True) / np.sqrt(d)
    floor = np.maximum(np.abs(Yref), rho)
    if dtype == "bf16":
        return ulp_bf16(Yref) + 4e-3 * floor
    return 1e-5 * floor


def summand_magnitude(X, d, radices, blocks, transpose=False):
    """Entrywise bound on the summands of every output: |X| through the stages with |blocks|."""
    from oracle import harp_oracle as ho
    ab = [np.abs(np.asarray(K, dtype=np.float64)) for K in blocks]
    fn = ho.apply_transpose_staged if transpose else ho.apply_staged
    return fn(np.abs(np.asarray(X, dtype=np.float64)), d, radices, ab, None)


def assert_parity(Y: np.ndarray, Yref: np.ndarray, dtype: str, what: str = "", mag=None, rho=None):
    assert Y.shape == Yref.shape, (Y.shape, Yref.shape)
    assert np.all(np.isfinite(Y)), f"{what}: non-finite output"
    err = np.abs(Y - Yref)
    tol = tolerance(Yref, dtype, rho)
    if mag is not None:
        tol = tol + 2e-6 * mag
    ratio = err / np.maximum(tol, 1e-300)
    worst = np.unravel_index(np.argmax(ratio), ratio.shape) if ratio.size else None
    if ratio.size and ratio[worst] > 1.0:
        raise AssertionError(
            f"{what}: |err|={err[worst]:.3e} > tol={tol[worst]:.3e} at {worst}, "
            f"ref={Yref[worst]:.6e} got={Y[worst]:.6e}; "
            f"normwise={np.linalg.norm(Y - Yref) / max(np.linalg.norm(Yref), 1e-300):.3e}")
    return float(ratio.max()) if ratio.size else 0.0
