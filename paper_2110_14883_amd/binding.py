"""ctypes binding of libtplinear.so: same names as the C ABI (include/tp_linear.h), argument
marshalling only.  Tensors are torch CUDA(ROCm) tensors used purely as device buffers: their
data_ptr(), row stride and dtype are handed to the library; nothing is computed here."""
from __future__ import annotations

import contextlib
import contextvars
import ctypes as C
import os
from dataclasses import dataclass

MODE_1D_COL, MODE_1D_ROW, MODE_2D, MODE_2P5D, MODE_3D, MODE_3D_GATHERED = 10, 11, 2, 25, 3, 33
EPI_NONE, EPI_BIAS, EPI_BIAS_GELU = 0, 1, 2
PASS_FWD, PASS_DX, PASS_DW, PASS_DX_PARTIALS, PASS_DW_PARTIALS = 0, 1, 2, 3, 4
DT_BF16, DT_F32 = 0, 1
MAX_STEPS = 16

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtplinear.so")
_lib = None


class TpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {tp_strerror(status)} (status {status})")


class _GridS(C.Structure):
    _fields_ = [("mode", C.c_int), ("q", C.c_int), ("d", C.c_int), ("p", C.c_int),
                ("ri", C.c_int), ("rj", C.c_int), ("rk", C.c_int)]


class _DimsS(C.Structure):
    _fields_ = [("M", C.c_int64), ("H", C.c_int64), ("F", C.c_int64)]


class _CBlk(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("ld", C.c_int64)]


class _OBlk(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("ld", C.c_int64), ("dtype", C.c_int)]


class _PlanOpts(C.Structure):
    _fields_ = [("tile", C.c_int), ("split_k", C.c_int), ("group_m", C.c_int), ("rotate", C.c_int), ("trim", C.c_int)]


# Launch-plan options handed to every *_ex call made inside `with plan_opts(...)` (tp_plan_opts_t; the
# library itself keeps no such state).  A context variable: each thread / task has its own.
_plan_opts: contextvars.ContextVar = contextvars.ContextVar("tp_plan_opts", default=None)


@contextlib.contextmanager
def plan_opts(tile: int = 0, split_k: int = 0, group_m: int = 0, rotate: int = 0, trim: int = 0):
    """tile: 0 auto, 1 = 256x256 (four-wave kernel), 2 = 128x256, 3 = 256x128, 4 = 128x128, 5 = 256x256 on the
    eight-wave kernel; split_k 0 auto, 1..8; group_m 0 auto, 1..64; rotate / trim: 0 auto (on), 1 on, 2 off."""
    token = _plan_opts.set(_PlanOpts(int(tile), int(split_k), int(group_m), int(rotate), int(trim)))
    try:
        yield
    finally:
        _plan_opts.reset(token)


def _opts():
    o = _plan_opts.get()
    return None if o is None else C.byref(o)


@dataclass(frozen=True)
class Grid:
    """1D: p = size, ri = rank.  2D: q, (ri, rj).  2.5D: q, d, (ri, rj, rk).  3D: p, (ri, rj, rk)."""
    mode: int
    q: int = 1
    d: int = 1
    p: int = 1
    ri: int = 0
    rj: int = 0
    rk: int = 0

    def _c(self) -> _GridS:
        return _GridS(self.mode, self.q, self.d, self.p, self.ri, self.rj, self.rk)


def lib() -> C.CDLL:
    """The loaded library.  No fallback: a missing build is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is not built; run `python -m paper_2110_14883_amd.build`")
        L = C.CDLL(_LIB_PATH)
        ip, i64p = C.POINTER(C.c_int), C.POINTER(C.c_int64)
        L.tp_block_map.restype = C.c_int
        L.tp_block_map.argtypes = [C.POINTER(_GridS), C.POINTER(_DimsS), C.c_int, ip, i64p, i64p, i64p,
                                   ip, ip, ip, ip, ip, ip, ip]
        po = C.POINTER(_PlanOpts)
        ws_args = [C.POINTER(_GridS), C.POINTER(_DimsS), C.c_int]
        fwd_args = [C.POINTER(_GridS), C.POINTER(_DimsS), C.c_int, C.POINTER(_CBlk), C.POINTER(_CBlk),
                    C.c_void_p, C.c_int, _OBlk, _OBlk, C.c_void_p, C.c_size_t, C.c_void_p]
        bwd_args = [C.POINTER(_GridS), C.POINTER(_DimsS), C.c_int, C.c_int,
                    C.POINTER(_CBlk), C.POINTER(_CBlk), C.POINTER(_CBlk), C.POINTER(_CBlk),
                    C.POINTER(_CBlk), C.POINTER(_CBlk), C.c_int, C.c_int, C.POINTER(_CBlk),
                    _OBlk, _OBlk, _OBlk, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        part_args = [C.POINTER(_GridS), C.POINTER(_DimsS), C.c_int, C.c_int, C.POINTER(_CBlk),
                     C.POINTER(_CBlk), C.POINTER(_OBlk), C.POINTER(_CBlk), C.POINTER(_OBlk),
                     C.c_void_p, C.c_size_t, C.c_void_p]
        L.tp_linear_workspace_size.restype = C.c_size_t
        L.tp_linear_workspace_size.argtypes = ws_args
        L.tp_linear_workspace_size_ex.restype = C.c_size_t
        L.tp_linear_workspace_size_ex.argtypes = ws_args + [po]
        L.tp_linear_fwd.restype = C.c_int
        L.tp_linear_fwd.argtypes = fwd_args
        L.tp_linear_fwd_ex.restype = C.c_int
        L.tp_linear_fwd_ex.argtypes = fwd_args + [po]
        L.tp_linear_fwd_static.restype = C.c_int
        L.tp_linear_fwd_static.argtypes = fwd_args[:9] + [C.c_void_p]
        L.tp_static_scratch_bytes.restype = C.c_size_t
        L.tp_static_scratch_bytes.argtypes = []
        L.tp_linear_bwd.restype = C.c_int
        L.tp_linear_bwd.argtypes = bwd_args
        L.tp_linear_bwd_ex.restype = C.c_int
        L.tp_linear_bwd_ex.argtypes = bwd_args + [po]
        L.tp_partials_map.restype = C.c_int
        L.tp_partials_map.argtypes = [C.POINTER(_GridS), C.POINTER(_DimsS), C.c_int, ip, i64p, i64p, i64p,
                                      ip, ip, ip, ip, ip, ip]
        L.tp_linear_bwd_partials.restype = C.c_int
        L.tp_linear_bwd_partials.argtypes = part_args
        L.tp_linear_bwd_partials_ex.restype = C.c_int
        L.tp_linear_bwd_partials_ex.argtypes = part_args + [po]
        L.tp_bias_act.restype = C.c_int
        L.tp_bias_act.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int, _OBlk, _OBlk, C.c_int64, C.c_int64, C.c_void_p]
        L.tp_dgelu.restype = C.c_int
        L.tp_dgelu.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                               C.c_int64, C.c_int64, C.c_void_p]
        L.tp_bias_grad.restype = C.c_int
        L.tp_bias_grad.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.tp_bias_grad_workspace_size.restype = C.c_size_t
        L.tp_bias_grad_workspace_size.argtypes = [C.c_int64, C.c_int64]
        L.tp_strerror.restype = C.c_char_p
        L.tp_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


EXPORTS = ("tp_block_map", "tp_linear_workspace_size", "tp_linear_workspace_size_ex", "tp_linear_fwd", "tp_linear_fwd_ex",
           "tp_linear_bwd", "tp_linear_bwd_ex", "tp_dgelu", "tp_partials_map", "tp_linear_bwd_partials",
           "tp_linear_bwd_partials_ex", "tp_bias_act", "tp_bias_grad", "tp_strerror", "tp_linear_fwd_static",
           "tp_static_scratch_bytes", "tp_bias_grad_workspace_size")


# ----------------------------------------------------------------------------- marshalling helpers
def _dims(dims) -> _DimsS:
    M, H, F = dims
    return _DimsS(int(M), int(H), int(F))


def _is_tensor(t) -> bool:
    return hasattr(t, "data_ptr")


def _ld(t) -> int:
    if t.dim() == 1:
        return int(t.shape[0])
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("blocks must be 2-D with unit column stride")
    return int(t.stride(0))


def _cblk(t) -> _CBlk:
    """torch tensor or (ptr, ld) pair -> tp_cblk_t."""
    if t is None:
        return _CBlk(None, 0)
    if _is_tensor(t):
        return _CBlk(t.data_ptr(), _ld(t))
    return _CBlk(int(t[0]) or None, int(t[1]))


def _cblk_array(blocks, n):
    if blocks is None:
        return None
    arr = (_CBlk * max(n, len(blocks), 1))()
    for i, b in enumerate(blocks):
        arr[i] = _cblk(b)
    return arr


def _oblk_array(blocks, n):
    if blocks is None:
        return None
    arr = (_OBlk * max(n, len(blocks), 1))()
    for i, b in enumerate(blocks):
        arr[i] = _oblk(b)
    return arr


def _cblk_ptr(t):
    return None if t is None else C.byref(_cblk(t))


def _oblk(t) -> _OBlk:
    """torch tensor, (ptr, ld, dtype) triple or None -> tp_oblk_t."""
    if t is None:
        return _OBlk(None, 0, 0)
    if _is_tensor(t):
        import torch
        if t.dtype == torch.float32:
            dt = DT_F32
        elif t.dtype == torch.bfloat16:
            dt = DT_BF16
        else:
            dt = 99                    # the library answers TP_ERR_DTYPE
        return _OBlk(t.data_ptr(), _ld(t), dt)
    return _OBlk(int(t[0]) or None, int(t[1]), int(t[2]))


def _ptr(t):
    if t is None:
        return None
    return t.data_ptr() if _is_tensor(t) else int(t)


def _ws(workspace):
    if workspace is None:
        return None, 0
    if _is_tensor(workspace):
        return workspace.data_ptr(), workspace.numel() * workspace.element_size()
    return int(workspace[0]), int(workspace[1])


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _check(status: int, where: str) -> None:
    if status != 0:
        raise TpError(status, where)


# ----------------------------------------------------------------------------- the ABI, same names
def tp_strerror(status: int) -> str:
    return lib().tp_strerror(int(status)).decode()


def tp_block_map(grid: Grid, dims, pass_: int) -> dict:
    n_steps, out_row, out_col, partial = C.c_int(), C.c_int(), C.c_int(), C.c_int()
    m, n, k = C.c_int64(), C.c_int64(), C.c_int64()
    arrs = [(C.c_int * MAX_STEPS)() for _ in range(4)]
    g, d = grid._c(), _dims(dims)
    st = lib().tp_block_map(C.byref(g), C.byref(d), int(pass_), C.byref(n_steps), C.byref(m), C.byref(n), C.byref(k),
                            arrs[0], arrs[1], arrs[2], arrs[3], C.byref(out_row), C.byref(out_col), C.byref(partial))
    _check(st, "tp_block_map")
    s = n_steps.value
    return dict(n_steps=s, m=m.value, n=n.value, k=k.value,
                a=[(arrs[0][i], arrs[1][i]) for i in range(s)], b=[(arrs[2][i], arrs[3][i]) for i in range(s)],
                out=(out_row.value, out_col.value), partial=bool(partial.value))


def tp_linear_workspace_size(grid: Grid, dims, pass_: int) -> int:
    g, d = grid._c(), _dims(dims)
    return int(lib().tp_linear_workspace_size_ex(C.byref(g), C.byref(d), int(pass_), _opts()))


def tp_linear_fwd(grid: Grid, dims, n_steps: int, x_blocks, w_blocks, bias, epi: int, y, preact=None,
                  workspace=None, stream=None) -> None:
    g, d = grid._c(), _dims(dims)
    ws, wsb = _ws(workspace)
    st = lib().tp_linear_fwd_ex(C.byref(g), C.byref(d), int(n_steps), _cblk_array(x_blocks, n_steps),
                                _cblk_array(w_blocks, n_steps), _ptr(bias), int(epi), _oblk(y), _oblk(preact),
                                ws, wsb, _stream(stream), _opts())
    _check(st, "tp_linear_fwd")


def tp_linear_fwd_static(grid: Grid, dims, n_steps: int, x_blocks, w_blocks, bias, epi: int, y, preact=None,
                         stream=None) -> None:
    """tp_linear_fwd without a workspace: K-split partials go to the library's built-in scratch array."""
    g, d = grid._c(), _dims(dims)
    st = lib().tp_linear_fwd_static(C.byref(g), C.byref(d), int(n_steps), _cblk_array(x_blocks, n_steps),
                                    _cblk_array(w_blocks, n_steps), _ptr(bias), int(epi), _oblk(y), _oblk(preact),
                                    _stream(stream))
    _check(st, "tp_linear_fwd_static")


def tp_static_scratch_bytes() -> int:
    return int(lib().tp_static_scratch_bytes())


def tp_linear_bwd(grid: Grid, dims, n_steps_dx: int = 0, n_steps_dw: int = 0, dy_own=None, preact_own=None,
                  da_row_blocks=None, w_blocks_dx=None, x_blocks_dw=None, da_col_blocks=None,
                  own_slot_dx: int = -1, own_slot_dw: int = -1, dgelu_preact=None,
                  dx=None, dw=None, da_own_out=None, db=None, workspace=None, stream=None) -> None:
    g, d = grid._c(), _dims(dims)
    ws, wsb = _ws(workspace)
    st = lib().tp_linear_bwd_ex(C.byref(g), C.byref(d), int(n_steps_dx), int(n_steps_dw),
                             _cblk_ptr(dy_own), _cblk_ptr(preact_own),
                             _cblk_array(da_row_blocks, n_steps_dx), _cblk_array(w_blocks_dx, n_steps_dx),
                             _cblk_array(x_blocks_dw, n_steps_dw), _cblk_array(da_col_blocks, n_steps_dw),
                             int(own_slot_dx), int(own_slot_dw), _cblk_ptr(dgelu_preact),
                             _oblk(dx), _oblk(dw), _oblk(da_own_out), _ptr(db), ws, wsb, _stream(stream), _opts())
    _check(st, "tp_linear_bwd")


def tp_dgelu(dy, preact, da, rows: int | None = None, cols: int | None = None, stream=None) -> None:
    if rows is None:
        rows, cols = int(dy.shape[0]), int(dy.shape[1])
    a, b, c = _cblk(dy), _cblk(preact), _cblk(da)
    st = lib().tp_dgelu(a.ptr, a.ld, b.ptr, b.ld, c.ptr, c.ld, int(rows), int(cols), _stream(stream))
    _check(st, "tp_dgelu")


def tp_partials_map(grid: Grid, dims, pass_: int) -> dict:
    n_steps, own_row, own_col = C.c_int(), C.c_int(), C.c_int()
    m, n, k = C.c_int64(), C.c_int64(), C.c_int64()
    arrs = [(C.c_int * MAX_STEPS)() for _ in range(4)]
    g, d = grid._c(), _dims(dims)
    st = lib().tp_partials_map(C.byref(g), C.byref(d), int(pass_), C.byref(n_steps), C.byref(m), C.byref(n), C.byref(k),
                               C.byref(own_row), C.byref(own_col), arrs[0], arrs[1], arrs[2], arrs[3])
    _check(st, "tp_partials_map")
    s = n_steps.value
    return dict(n_steps=s, m=m.value, n=n.value, k=k.value, own=(own_row.value, own_col.value),
                other=[(arrs[0][i], arrs[1][i]) for i in range(s)], out=[(arrs[2][i], arrs[3][i]) for i in range(s)])


def tp_linear_bwd_partials(grid: Grid, dims, da_own, w_blocks_dx=None, dx_partials=None, x_blocks_dw=None,
                           dw_partials=None, workspace=None, stream=None) -> None:
    g, d = grid._c(), _dims(dims)
    ws, wsb = _ws(workspace)
    n_dx = 0 if w_blocks_dx is None else len(w_blocks_dx)
    n_dw = 0 if x_blocks_dw is None else len(x_blocks_dw)
    if (dx_partials is not None and len(dx_partials) != n_dx) or (dw_partials is not None and len(dw_partials) != n_dw):
        raise ValueError("one output block per operand block")
    st = lib().tp_linear_bwd_partials_ex(C.byref(g), C.byref(d), n_dx, n_dw, _cblk_ptr(da_own),
                                      _cblk_array(w_blocks_dx, n_dx), _oblk_array(dx_partials, n_dx),
                                      _cblk_array(x_blocks_dw, n_dw), _oblk_array(dw_partials, n_dw),
                                      ws, wsb, _stream(stream), _opts())
    _check(st, "tp_linear_bwd_partials")


def tp_bias_act(c, bias, epi: int, y, preact=None, rows: int | None = None, cols: int | None = None, stream=None) -> None:
    if rows is None:
        rows, cols = int(c.shape[0]), int(c.shape[1])
    ptr, ld = (c.data_ptr(), _ld(c)) if _is_tensor(c) else (int(c[0]), int(c[1]))
    st = lib().tp_bias_act(ptr or None, ld, _ptr(bias), int(epi), _oblk(y), _oblk(preact), int(rows), int(cols), _stream(stream))
    _check(st, "tp_bias_act")


def tp_bias_grad(da, db, rows: int | None = None, cols: int | None = None, workspace=None, stream=None) -> None:
    if rows is None:
        rows, cols = int(da.shape[0]), int(da.shape[1])
    a = _cblk(da)
    ws, wsb = _ws(workspace)
    _check(lib().tp_bias_grad(a.ptr, a.ld, int(rows), int(cols), _ptr(db), ws, wsb, _stream(stream)), "tp_bias_grad")


def tp_bias_grad_workspace_size(rows: int, cols: int) -> int:
    return int(lib().tp_bias_grad_workspace_size(int(rows), int(cols)))
