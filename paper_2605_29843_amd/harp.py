"""ctypes binding of libharp.so -- argument marshalling only.

Every step of the rotation path runs inside the HIP library; this module converts Python
arguments into the C ABI of ``include/harp.h`` (same names) and raises on error codes.
PyTorch is used for device memory (``tensor.data_ptr()``) and the current HIP stream, and
for nothing else.  Importing this module loads the shared library and raises ImportError
when it has not been built (``python -m paper_2605_29843_amd.build``): there is no CPU or
PyTorch fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
# PyTorch ships its own copy of the HIP runtime (same soname).  It must be loaded before
# libharp.so so that both resolve to ONE runtime instance: device pointers and streams
# created by PyTorch are then valid inside the library.
import torch  # noqa: F401  (import order matters)

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libharp.so")

HARP_OK, HARP_ERR_INVALID_ARG, HARP_ERR_BAD_SCHEDULE, HARP_ERR_NOT_ORTHOGONAL, \
    HARP_ERR_UNSUPPORTED, HARP_ERR_OOM, HARP_ERR_DEVICE = range(7)
HARP_F32, HARP_BF16 = 0, 1
HARP_VALIDATE_ORTHO, HARP_BLOCKS_ON_DEVICE, HARP_THETA_IN_KERNEL, HARP_F32_INTERMEDIATES = 1, 2, 4, 8
HARP_ALGO_AUTO, HARP_ALGO_GENERIC, HARP_ALGO_FUSED, HARP_ALGO_SPLIT = 0, 1, 2, 3
HARP_MAX_RADIX, HARP_MAX_STAGES = 64, 64
HARP_MIXER_IDENTITY, HARP_MIXER_HADAMARD, HARP_MIXER_CUSTOM = 0, 1, 2

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_29843_amd.build` "
                      "(the HARP path has no fallback implementation)")
lib = C.CDLL(LIB_PATH)

_vp, _i64, _i32, _u32, _sz = C.c_void_p, C.c_int64, C.c_int32, C.c_uint32, C.c_size_t
_SIGS = {
    "harp_plan_create": (_i32, [C.POINTER(_vp), _i64, _i32, C.POINTER(_i32), C.POINTER(_vp), _vp, _u32]),
    "harp_plan_destroy": (_i32, [_vp]),
    "harp_blocks_from_theta": (_i32, [_i64, _i32, C.POINTER(_i32), C.POINTER(_vp), C.POINTER(_i32),
                                      C.POINTER(_vp), C.POINTER(_vp)]),
    "harp_kronecker_blocks": (_i32, [_i32, _vp, _i64, _i32, C.POINTER(_i32), C.POINTER(_vp),
                                     C.POINTER(_i32), C.POINTER(_vp)]),
    "harp_plan_create_kronecker": (_i32, [C.POINTER(_vp), _i32, _vp, _i64, _i32, C.POINTER(_i32),
                                          C.POINTER(_vp), _vp, _u32]),
    "harp_plan_tied_slices": (_i32, [_vp]),
    "harp_plan_theta_in_kernel": (_i32, [_vp]),
    "harp_plan_create_from_theta": (_i32, [C.POINTER(_vp), _i64, _i32, C.POINTER(_i32), C.POINTER(_vp),
                                           C.POINTER(_i32), C.POINTER(_vp), _vp, _u32]),
    "harp_theta_quantize_int8": (_i32, [_i64, _i32, C.POINTER(_i32), C.POINTER(_vp), C.POINTER(_vp),
                                        C.POINTER(_vp)]),
    "harp_theta_dequantize_int8": (_i32, [_i64, _i32, C.POINTER(_i32), C.POINTER(_vp), C.POINTER(_vp),
                                          C.POINTER(_vp)]),
    "harp_plan_create_from_theta_int8": (_i32, [C.POINTER(_vp), _i64, _i32, C.POINTER(_i32),
                                                C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_i32),
                                                C.POINTER(_vp), _vp, _u32]),
    "harp_apply": (_i32, [_vp, _vp, _i64, _vp, _i64, _i64, _i32, _vp]),
    "harp_apply_transpose": (_i32, [_vp, _vp, _i64, _vp, _i64, _i64, _i32, _vp]),
    "harp_apply_noalloc": (_i32, [_vp, _vp, _i64, _vp, _i64, _i64, _i32, _i32, _vp]),
    "harp_apply_noalloc_max_rows": (_i64, [_vp]),
    "harp_rotate_weight_workspace_size": (_i32, [_vp, _vp, _i64, _i64, _i32, C.POINTER(_sz)]),
    "harp_rotate_weight": (_i32, [_vp, _vp, _vp, _i64, _vp, _i64, _i64, _i64, _i32, _vp, _sz, _vp]),
    "harp_rotate_weight_inverse": (_i32, [_vp, _vp, _vp, _i64, _vp, _i64, _i64, _i64, _i32, _vp, _sz, _vp]),
    "harp_grad_blocks_workspace_size": (_i32, [_vp, _i64, C.POINTER(_sz)]),
    "harp_grad_blocks": (_i32, [_vp, _vp, _i64, _vp, _i64, _i64, _i32, C.POINTER(_vp), _vp, _i64, _vp,
                                _sz, _vp]),
    "harp_greedy_schedule": (_i32, [_i64, _i32, _i32, C.POINTER(_i32), C.POINTER(_i32)]),
    "harp_plan_dim": (_i64, [_vp]),
    "harp_plan_num_stages": (_i32, [_vp]),
    "harp_plan_param_count": (_i64, [_vp]),
    "harp_plan_param_bytes": (_i64, [_vp]),
    "harp_plan_set_algo": (_i32, [_vp, _i32]),
    "harp_plan_set_rows_per_tile": (_i32, [_vp, _i32]),
    "harp_plan_kernel_name": (C.c_char_p, [_vp, _i64, _i32]),
    "harp_status_string": (C.c_char_p, [_i32]),
    "harp_version": (C.c_char_p, []),
}
EXPORTS = tuple(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)          # AttributeError here = the library lacks a declared symbol
    _f.restype, _f.argtypes = _res, _args


class HarpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        msg = lib.harp_status_string(int(status)).decode()
        super().__init__(f"{where}: {msg} (status {int(status)})")


def _check(status: int, where: str) -> None:
    if status != HARP_OK:
        raise HarpError(status, where)


def harp_status_string(status: int) -> str:
    return lib.harp_status_string(int(status)).decode()


def harp_version() -> str:
    return lib.harp_version().decode()


def harp_greedy_schedule(d: int, b_base: int = 8, b_max: int = 8) -> list[int]:
    out = (_i32 * HARP_MAX_STAGES)()
    m = _i32(0)
    _check(lib.harp_greedy_schedule(int(d), int(b_base), int(b_max), out, C.byref(m)),
           "harp_greedy_schedule")
    return [int(out[i]) for i in range(m.value)]


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return HARP_F32
    if t.dtype == torch.bfloat16:
        return HARP_BF16
    raise TypeError(f"unsupported dtype {t.dtype}; expected float32 or bfloat16")


def _stream_ptr(stream) -> int:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _on_stream(t, stream):
    """A tensor this module allocated (with the caching allocator, i.e. on the CURRENT stream) is
    about to be used by kernels on `stream`: tell the allocator, so that the block is not handed
    to other work on the current stream while those kernels are still running."""
    import torch
    if t is not None and stream is not None and stream != torch.cuda.current_stream():
        t.record_stream(stream)
    return t


def _rowmajor_2d(t, what: str):
    if t.dim() != 2 or t.stride(1) != 1 or not t.is_cuda:
        raise ValueError(f"{what} must be a 2-D device tensor with unit inner stride")
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def _theta_args(d, radices, thetas, mixers, keep):
    """ctypes arrays for the (theta, mixer_kinds, mixers) arguments.  thetas[t] / mixers[t]:
    None, or a host array; mixers[t] may also be "identity" or "hadamard"."""
    m = len(radices)
    th = (_vp * max(m, 1))()
    kinds = (_i32 * max(m, 1))()
    mx = (_vp * max(m, 1))()
    for t, b in enumerate(radices):
        a = None if thetas is None else thetas[t]
        if a is None:
            th[t] = None
        else:
            a = np.ascontiguousarray(a, dtype=np.float32)
            if a.size != (d // b) * (b * (b - 1) // 2):
                raise ValueError(f"theta[{t}] must hold D_t * b (b - 1) / 2 values")
            keep.append(a)
            th[t] = a.ctypes.data
        g = None if mixers is None else mixers[t]
        if g is None or (isinstance(g, str) and g == "hadamard"):
            kinds[t], mx[t] = HARP_MIXER_HADAMARD, None
        elif isinstance(g, str) and g == "identity":
            kinds[t], mx[t] = HARP_MIXER_IDENTITY, None
        else:
            g = np.ascontiguousarray(g, dtype=np.float32)
            if g.shape != (b, b):
                raise ValueError(f"mixers[{t}] must be {b} x {b}")
            keep.append(g)
            kinds[t], mx[t] = HARP_MIXER_CUSTOM, g.ctypes.data
    return th, kinds, mx


def harp_blocks_from_theta(d: int, radices, thetas=None, mixers=None) -> list:
    """Host blocks B = Q(theta) G per stage, float32 arrays [D_t, b_t, b_t]."""
    radices = [int(b) for b in radices]
    m = len(radices)
    keep = []
    th, kinds, mx = _theta_args(int(d), radices, thetas, mixers, keep)
    outs = [np.empty((max(int(d) // b, 0), b, b), dtype=np.float32) for b in radices]
    op = (_vp * max(m, 1))(*[o.ctypes.data for o in outs])
    rad = (_i32 * max(m, 1))(*radices)
    _check(lib.harp_blocks_from_theta(int(d), m, rad, th, kinds, mx, op), "harp_blocks_from_theta")
    return outs


def _npar(d, b):
    return (int(d) // b) * (b * (b - 1) // 2)


def harp_theta_quantize_int8(d: int, radices, thetas):
    """(codes, scales) per stage: int8 arrays [D_t, p_t] and float32 arrays [D_t]."""
    radices = [int(b) for b in radices]
    m = len(radices)
    ins = [np.ascontiguousarray(thetas[t], dtype=np.float32) for t in range(m)]
    for t, b in enumerate(radices):
        if ins[t].size != _npar(d, b):
            raise ValueError(f"theta[{t}] must hold D_t * b (b - 1) / 2 values")
    codes = [np.empty((int(d) // b, b * (b - 1) // 2), dtype=np.int8) for b in radices]
    scales = [np.empty(int(d) // b, dtype=np.float32) for b in radices]
    rad = (_i32 * max(m, 1))(*radices)
    ip = (_vp * max(m, 1))(*[a.ctypes.data for a in ins])
    cp = (_vp * max(m, 1))(*[a.ctypes.data for a in codes])
    sp = (_vp * max(m, 1))(*[a.ctypes.data for a in scales])
    _check(lib.harp_theta_quantize_int8(int(d), m, rad, ip, cp, sp), "harp_theta_quantize_int8")
    return codes, scales


def _int8_args(d, radices, codes, scales, keep):
    m = len(radices)
    cs = [np.ascontiguousarray(codes[t], dtype=np.int8) for t in range(m)]
    ss = [np.ascontiguousarray(scales[t], dtype=np.float32) for t in range(m)]
    for t, b in enumerate(radices):
        if cs[t].size != _npar(d, b) or ss[t].size != int(d) // b:
            raise ValueError(f"codes[{t}] / scales[{t}] have the wrong size")
    keep.extend(cs + ss)
    return ((_vp * max(m, 1))(*[a.ctypes.data for a in cs]),
            (_vp * max(m, 1))(*[a.ctypes.data for a in ss]))


def harp_theta_dequantize_int8(d: int, radices, codes, scales) -> list:
    """theta ~ scale * code per stage, float32 arrays [D_t, p_t]."""
    radices = [int(b) for b in radices]
    m = len(radices)
    keep = []
    cp, sp = _int8_args(d, radices, codes, scales, keep)
    outs = [np.empty((int(d) // b, b * (b - 1) // 2), dtype=np.float32) for b in radices]
    op = (_vp * max(m, 1))(*[a.ctypes.data for a in outs])
    rad = (_i32 * max(m, 1))(*radices)
    _check(lib.harp_theta_dequantize_int8(int(d), m, rad, cp, sp, op), "harp_theta_dequantize_int8")
    return outs


def harp_kronecker_blocks(table, n2: int, radices2, blocks2):
    """(radices, blocks) of the Mixed-Radix processor equal to (table / sqrt(K)) (x) T_{n2}."""
    table = np.ascontiguousarray(table, dtype=np.float32)
    K = int(table.shape[0])
    if table.shape != (K, K):
        raise ValueError("table must be square")
    radices2 = [int(b) for b in radices2]
    m2 = len(radices2)
    ins = [np.ascontiguousarray(blocks2[t], dtype=np.float32) for t in range(m2)]
    outs = [np.empty((K * (int(n2) // b), b, b), dtype=np.float32) for b in radices2]
    outs.append(np.empty((int(n2), K, K), dtype=np.float32))
    rad2 = (_i32 * max(m2, 1))(*radices2)
    ip = (_vp * max(m2, 1))(*[a.ctypes.data for a in ins])
    op = (_vp * (m2 + 1))(*[o.ctypes.data for o in outs])
    rout = (_i32 * (m2 + 1))()
    _check(lib.harp_kronecker_blocks(K, table.ctypes.data, int(n2), m2, rad2, ip, rout, op),
           "harp_kronecker_blocks")
    return [int(rout[i]) for i in range(m2 + 1)], outs


class Plan:
    """Owner of a ``harp_plan_t*``.  ``harp_plan_create`` with host numpy arrays."""

    def __init__(self, d: int, radices, blocks, signs=None, flags: int = 0):
        radices = [int(b) for b in radices]
        m = len(radices)
        self._keep = []
        rad = (_i32 * max(m, 1))(*radices)
        ptrs = (_vp * max(m, 1))()
        for t in range(m):
            if blocks[t] is None:
                ptrs[t] = None
                continue
            a = np.ascontiguousarray(blocks[t], dtype=np.float32)
            self._keep.append(a)
            ptrs[t] = a.ctypes.data
        sp = None
        if signs is not None:
            s = np.ascontiguousarray(signs, dtype=np.int8)
            self._keep.append(s)
            sp = s.ctypes.data
        self._h = _vp(None)
        self.d, self.radices = int(d), radices
        _check(lib.harp_plan_create(C.byref(self._h), int(d), m, rad, ptrs, sp, int(flags)),
               "harp_plan_create")
        self._keep = []   # the plan copied everything it needs

    @classmethod
    def from_theta(cls, d: int, radices, thetas=None, mixers=None, signs=None, flags: int = 0):
        """``harp_plan_create_from_theta``: rotation parameters instead of dense blocks."""
        self = cls.__new__(cls)
        radices = [int(b) for b in radices]
        m = len(radices)
        keep = []
        th, kinds, mx = _theta_args(int(d), radices, thetas, mixers, keep)
        rad = (_i32 * max(m, 1))(*radices)
        sp = None
        if signs is not None:
            s = np.ascontiguousarray(signs, dtype=np.int8)
            keep.append(s)
            sp = s.ctypes.data
        self._h = _vp(None)
        self._keep = []
        self.d, self.radices = int(d), radices
        _check(lib.harp_plan_create_from_theta(C.byref(self._h), int(d), m, rad, th, kinds, mx, sp,
                                               int(flags)), "harp_plan_create_from_theta")
        return self

    @classmethod
    def from_theta_int8(cls, d: int, radices, codes, scales, mixers=None, signs=None, flags: int = 0):
        """``harp_plan_create_from_theta_int8``: int8 codes and per-block scales."""
        self = cls.__new__(cls)
        radices = [int(b) for b in radices]
        m = len(radices)
        keep = []
        _, kinds, mx = _theta_args(int(d), radices, None, mixers, keep)
        cp, scp = _int8_args(int(d), radices, codes, scales, keep)
        rad = (_i32 * max(m, 1))(*radices)
        sp = None
        if signs is not None:
            s = np.ascontiguousarray(signs, dtype=np.int8)
            keep.append(s)
            sp = s.ctypes.data
        self._h = _vp(None)
        self._keep = []
        self.d, self.radices = int(d), radices
        _check(lib.harp_plan_create_from_theta_int8(C.byref(self._h), int(d), m, rad, cp, scp, kinds,
                                                    mx, sp, int(flags)),
               "harp_plan_create_from_theta_int8")
        return self

    @classmethod
    def kronecker(cls, table, n2: int, radices2, blocks2, signs=None, flags: int = 0):
        """``harp_plan_create_kronecker``: (table / sqrt(K)) (x) T_{n2} with tied parameters."""
        self = cls.__new__(cls)
        table = np.ascontiguousarray(table, dtype=np.float32)
        K = int(table.shape[0])
        if table.shape != (K, K):
            raise ValueError("table must be square")
        radices2 = [int(b) for b in radices2]
        m2 = len(radices2)
        ins = [np.ascontiguousarray(blocks2[t], dtype=np.float32) for t in range(m2)]
        rad2 = (_i32 * max(m2, 1))(*radices2)
        ip = (_vp * max(m2, 1))(*[a.ctypes.data for a in ins])
        sp = None
        if signs is not None:
            s = np.ascontiguousarray(signs, dtype=np.int8)
            if s.size != K * int(n2):
                raise ValueError("signs must hold K * n2 values")
            sp = s.ctypes.data
        self._h = _vp(None)
        self._keep = []
        self.d, self.radices = K * int(n2), radices2 + [K]
        _check(lib.harp_plan_create_kronecker(C.byref(self._h), K, table.ctypes.data, int(n2), m2, rad2,
                                              ip, sp, int(flags)), "harp_plan_create_kronecker")
        return self

    def tied_slices(self) -> int:
        return int(lib.harp_plan_tied_slices(self._h))

    def theta_in_kernel(self) -> bool:
        return int(lib.harp_plan_theta_in_kernel(self._h)) == 1

    # -- lifetime
    def destroy(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib.harp_plan_destroy(self._h)
            self._h = _vp(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    # -- introspection / tuning
    def dim(self) -> int:
        return int(lib.harp_plan_dim(self._h))

    def num_stages(self) -> int:
        return int(lib.harp_plan_num_stages(self._h))

    def param_count(self) -> int:
        return int(lib.harp_plan_param_count(self._h))

    def param_bytes(self) -> int:
        return int(lib.harp_plan_param_bytes(self._h))

    def set_algo(self, algo: int) -> None:
        _check(lib.harp_plan_set_algo(self._h, int(algo)), "harp_plan_set_algo")

    def set_rows_per_tile(self, rows: int) -> None:
        _check(lib.harp_plan_set_rows_per_tile(self._h, int(rows)), "harp_plan_set_rows_per_tile")

    def kernel_name(self, n: int = 1, dtype_code: int = HARP_BF16) -> str:
        return lib.harp_plan_kernel_name(self._h, int(n), int(dtype_code)).decode()


def harp_plan_create(d, radices, blocks, signs=None, flags=0) -> Plan:
    return Plan(d, radices, blocks, signs, flags)


def harp_plan_destroy(plan: Plan) -> None:
    plan.destroy()


def _apply(fn, name, plan: Plan, X, Y=None, stream=None):
    import torch
    if Y is None:
        Y = _on_stream(torch.empty_like(X), stream)
    if X.shape != Y.shape or X.dtype != Y.dtype:
        raise ValueError("X and Y must have the same shape and dtype")
    ldx, ldy = _rowmajor_2d(X, "X"), _rowmajor_2d(Y, "Y")
    if X.shape[1] != plan.d:
        raise ValueError(f"X has {X.shape[1]} columns, plan dimension is {plan.d}")
    _check(fn(plan.handle, X.data_ptr(), ldx, Y.data_ptr(), ldy, X.shape[0], _dtype_code(X),
              _stream_ptr(stream)), name)
    return Y


def harp_apply(plan: Plan, X, Y=None, stream=None):
    """Y = X U on device tensors (float32 or bfloat16); allocates Y when not given."""
    return _apply(lib.harp_apply, "harp_apply", plan, X, Y, stream)


def harp_apply_transpose(plan: Plan, X, Y=None, stream=None):
    """Y = X U^T."""
    return _apply(lib.harp_apply_transpose, "harp_apply_transpose", plan, X, Y, stream)


def harp_apply_noalloc(plan: Plan, X, Y, transpose: bool = False, stream=None):
    """``harp_apply`` / ``harp_apply_transpose`` without any allocation: Y must be given."""
    if X.shape != Y.shape or X.dtype != Y.dtype:
        raise ValueError("X and Y must have the same shape and dtype")
    ldx, ldy = _rowmajor_2d(X, "X"), _rowmajor_2d(Y, "Y")
    if X.shape[1] != plan.d:
        raise ValueError(f"X has {X.shape[1]} columns, plan dimension is {plan.d}")
    _check(lib.harp_apply_noalloc(plan.handle, X.data_ptr(), ldx, Y.data_ptr(), ldy, X.shape[0],
                                  _dtype_code(X), 1 if transpose else 0, _stream_ptr(stream)),
           "harp_apply_noalloc")
    return Y


def harp_apply_noalloc_max_rows(plan: Plan) -> int:
    return int(lib.harp_apply_noalloc_max_rows(plan.handle))


def harp_grad_blocks_workspace_size(plan, n: int) -> int:
    b = _sz(0)
    _check(lib.harp_grad_blocks_workspace_size(plan.handle, int(n), C.byref(b)),
           "harp_grad_blocks_workspace_size")
    return int(b.value)


def harp_grad_blocks(plan, X, G, want_dX: bool = True, workspace=None, stream=None):
    """(dK, dX): gradients of a loss with dL/dY = G through Y = X U.  dK[t] is a float32 device
    tensor [D_t, b_t, b_t]; dX has the shape and type of X (None when want_dX is false)."""
    import torch
    if X.shape != G.shape or X.dtype != G.dtype:
        raise ValueError("X and G must have the same shape and dtype")
    ldx, ldg = _rowmajor_2d(X, "X"), _rowmajor_2d(G, "G")
    n, d = X.shape
    if d != plan.d:
        raise ValueError("X has the wrong number of columns")
    dt = _dtype_code(X)
    dK = [_on_stream(torch.empty((plan.d // b, b, b), dtype=torch.float32, device=X.device), stream)
          for b in plan.radices]
    dX = _on_stream(torch.empty_like(X), stream) if want_dX else None
    need = harp_grad_blocks_workspace_size(plan, n)
    if workspace is None and need:
        workspace = _on_stream(torch.empty(need, dtype=torch.uint8, device=X.device), stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    ptrs = (_vp * max(len(dK), 1))(*[t.data_ptr() for t in dK])
    _check(lib.harp_grad_blocks(plan.handle, X.data_ptr(), ldx, G.data_ptr(), ldg, n, dt, ptrs,
                                dX.data_ptr() if dX is not None else None,
                                _rowmajor_2d(dX, "dX") if dX is not None else 0, ws_ptr, ws_bytes,
                                _stream_ptr(stream)), "harp_grad_blocks")
    return dK, dX


def harp_rotate_weight_workspace_size(plan_U, plan_V, d_out, d_in, dtype_code) -> int:
    b = _sz(0)
    _check(lib.harp_rotate_weight_workspace_size(plan_U.handle if plan_U else None,
                                                 plan_V.handle if plan_V else None,
                                                 int(d_out), int(d_in), int(dtype_code), C.byref(b)),
           "harp_rotate_weight_workspace_size")
    return int(b.value)


def _rotate(fn, name, plan_U, plan_V, W, Wout=None, workspace=None, stream=None):
    import torch
    if Wout is None:
        Wout = _on_stream(torch.empty_like(W), stream)
    if W.shape != Wout.shape or W.dtype != Wout.dtype:
        raise ValueError("W and Wout must have the same shape and dtype")
    ldw, ldo = _rowmajor_2d(W, "W"), _rowmajor_2d(Wout, "Wout")
    d_out, d_in = W.shape
    dt = _dtype_code(W)
    need = harp_rotate_weight_workspace_size(plan_U, plan_V, d_out, d_in, dt)
    if workspace is None and need:
        workspace = _on_stream(torch.empty(need, dtype=torch.uint8, device=W.device), stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(fn(plan_U.handle if plan_U else None, plan_V.handle if plan_V else None,
              W.data_ptr(), ldw, Wout.data_ptr(), ldo, d_out, d_in, dt, ws_ptr, ws_bytes,
              _stream_ptr(stream)), name)
    return Wout


def harp_rotate_weight(plan_U, plan_V, W, Wout=None, workspace=None, stream=None):
    """Wout = U_U^T W U_V."""
    return _rotate(lib.harp_rotate_weight, "harp_rotate_weight", plan_U, plan_V, W, Wout,
                   workspace, stream)


def harp_rotate_weight_inverse(plan_U, plan_V, W, Wout=None, workspace=None, stream=None):
    """Wout = U_U W U_V^T."""
    return _rotate(lib.harp_rotate_weight_inverse, "harp_rotate_weight_inverse", plan_U, plan_V,
                   W, Wout, workspace, stream)
