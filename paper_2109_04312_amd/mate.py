"""ctypes binding over libmate.so (the C ABI of include/mate.h).  Argument marshalling only.

The raw entry points are exposed under their C names (`mate_build_segments`, ...) taking
integer addresses; the snake-case helpers below take torch tensors, allocate outputs with
torch (device memory + current stream are all torch is used for) and raise on any non-zero
status.  There is no fallback: if the library is missing this module raises on import.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MATE_LIBRARY", os.path.join(_HERE, "libmate.so"))

MATE_OK = 0
MATE_ERR_NULL, MATE_ERR_SHAPE, MATE_ERR_UNSUPPORTED = -1, -2, -3
MATE_ERR_WORKSPACE, MATE_ERR_BAD_ID, MATE_ERR_HIP = -4, -5, -6
MATE_F32, MATE_BF16 = 0, 1
MATE_TOK_LOCAL, MATE_TOK_GLOBAL, MATE_TOK_PAD = 0, 1, 2
MATE_HEAD_ROW, MATE_HEAD_COL = 0, 1
MATE_MAX_N, MATE_MAX_HEADS, MATE_HEAD_DIM = 16384, 256, 64

EXPORTS = ["mate_segments_bytes", "mate_workspace_bytes", "mate_build_segments",
           "mate_build_segments_bucketed", "mate_cell_positions", "mate_segments_export", "mate_segments_export_windows", "mate_attn_fwd", "mate_attn_bwd", "mate_dense_workspace_bytes",
           "mate_attn_fwd_dense", "mate_attn_bwd_dense", "mate_attn_bwd_dense_static", "mate_attn_prefers_dense", "mate_segments_status", "mate_qkv_project", "mate_out_project", "mate_project_bwd_workspace_bytes", "mate_qkv_project_bwd", "mate_out_project_bwd", "mate_profile_kernel",
           "mate_probe_mfma", "mate_status_string"]
MATE_KERNEL_NONE, MATE_KERNEL_BUILD, MATE_KERNEL_FWD = 0, 1, 2
MATE_KERNEL_BWD_DQ, MATE_KERNEL_BWD_DKV = 3, 4
MATE_KERNEL_FWD_DENSE, MATE_KERNEL_BWD_DQ_DENSE, MATE_KERNEL_BWD_DKV_DENSE = 5, 6, 7
MATE_KERNEL_QKV_PROJECT, MATE_KERNEL_OUT_PROJECT = 8, 9
MATE_KERNEL_QKV_PROJECT_DGRAD, MATE_KERNEL_QKV_PROJECT_WGRAD = 10, 11
MATE_KERNEL_OUT_PROJECT_DGRAD, MATE_KERNEL_OUT_PROJECT_WGRAD = 12, 13
MATE_DENSE_MAX_N = 1024
MATE_DENSE_PREFERRED_MAX_N = 256

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2109_04312_amd.build` "
                      "(there is no CPU fallback)")
_lib = C.CDLL(LIB_PATH)

_p, _i, _sz, _f = C.c_void_p, C.c_int, C.c_size_t, C.c_float
_lib.mate_segments_bytes.restype = _sz
_lib.mate_segments_bytes.argtypes = [_i, _i]
_lib.mate_workspace_bytes.restype = _sz
_lib.mate_workspace_bytes.argtypes = [_i, _i, _i, _i, _i, _i]
_lib.mate_build_segments.restype = _i
_lib.mate_build_segments.argtypes = [_p, _p, _p, _i, _i, _p, _p]
_lib.mate_build_segments_bucketed.restype = _i
_lib.mate_build_segments_bucketed.argtypes = [_p, _p, _p, _i, _i, _i, _i, _p, _p]
_lib.mate_segments_export_windows.restype = _i
_lib.mate_segments_export_windows.argtypes = [_p, _i, _i, _i, _p, _p]
_lib.mate_cell_positions.restype = _i
_lib.mate_cell_positions.argtypes = [_p, _p, _p, _i, _i, _p, _p]
_lib.mate_segments_export.restype = _i
_lib.mate_segments_export.argtypes = [_p, _i, _i, _i, _p, _p, _p, _p, _p, _p]
_lib.mate_attn_fwd.restype = _i
_lib.mate_attn_fwd.argtypes = [_p, _p, _p, _p, _p, _i, _i, _i, _i, _i, _f, _p, _p, _p, _sz, _p]
_lib.mate_attn_bwd.restype = _i
_lib.mate_attn_bwd.argtypes = [_p, _p, _p, _p, _p, _p, _p, _p, _i, _i, _i, _i, _i, _f,
                               _p, _p, _p, _p, _sz, _p]
_lib.mate_dense_workspace_bytes.restype = _sz
_lib.mate_dense_workspace_bytes.argtypes = [_i, _i, _i]
_lib.mate_attn_prefers_dense.restype = _i
_lib.mate_attn_prefers_dense.argtypes = [_i, _i, _i, _i]
_lib.mate_segments_status.restype = _i
_lib.mate_segments_status.argtypes = [_p, _i, _i, _p]
_lib.mate_attn_fwd_dense.restype = _i
_lib.mate_attn_fwd_dense.argtypes = [_p, _p, _p, _p, _p, _p, _p, _i, _i, _i, _i, _i, _f, _p, _p, _p]
_lib.mate_attn_bwd_dense.restype = _i
_lib.mate_attn_bwd_dense.argtypes = [_p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _i, _i, _i, _i, _i, _f,
                                     _p, _p, _p, _p, _sz, _p]
_lib.mate_attn_bwd_dense_static.restype = _i
_lib.mate_attn_bwd_dense_static.argtypes = [_p, _p, _p, _p, _p, _p, _p, _p, _p, _p, _i, _i, _i, _i, _i, _f,
                                            _p, _p, _p, _p]
_lib.mate_qkv_project.restype = _i
_lib.mate_qkv_project.argtypes = [_p, _p, _p, _p, _i, _i, _i, _i, _i, _p, _p, _p, _p]
_lib.mate_out_project.restype = _i
_lib.mate_out_project.argtypes = [_p, _p, _p, _p, _i, _i, _i, _i, _i, _p, _p]
_lib.mate_project_bwd_workspace_bytes.restype = _sz
_lib.mate_project_bwd_workspace_bytes.argtypes = [_i, _i, _i, _i]
_lib.mate_qkv_project_bwd.restype = _i
_lib.mate_qkv_project_bwd.argtypes = [_p, _p, _p, _p, _p, _p, _i, _i, _i, _i, _i, _p, _p, _p, _p, _sz, _p]
_lib.mate_out_project_bwd.restype = _i
_lib.mate_out_project_bwd.argtypes = [_p, _p, _p, _p, _i, _i, _i, _i, _i, _p, _p, _p, _p, _sz, _p]
_lib.mate_profile_kernel.restype = _i
_lib.mate_profile_kernel.argtypes = [_i, _p, _p]
_lib.mate_probe_mfma.restype = _i
_lib.mate_probe_mfma.argtypes = [_p, _sz, _i, _i, C.POINTER(C.c_double), _p]
_lib.mate_status_string.restype = C.c_char_p
_lib.mate_status_string.argtypes = [_i]

mate_segments_bytes = _lib.mate_segments_bytes
mate_workspace_bytes = _lib.mate_workspace_bytes
mate_build_segments = _lib.mate_build_segments
mate_segments_export = _lib.mate_segments_export
mate_cell_positions = _lib.mate_cell_positions
mate_build_segments_bucketed = _lib.mate_build_segments_bucketed
mate_segments_export_windows = _lib.mate_segments_export_windows
mate_attn_fwd = _lib.mate_attn_fwd
mate_attn_bwd = _lib.mate_attn_bwd
mate_profile_kernel = _lib.mate_profile_kernel
mate_probe_mfma = _lib.mate_probe_mfma
mate_dense_workspace_bytes = _lib.mate_dense_workspace_bytes
mate_attn_prefers_dense = _lib.mate_attn_prefers_dense
mate_segments_status = _lib.mate_segments_status
mate_attn_fwd_dense = _lib.mate_attn_fwd_dense
mate_attn_bwd_dense = _lib.mate_attn_bwd_dense
mate_attn_bwd_dense_static = _lib.mate_attn_bwd_dense_static
MATE_STATIC_SCRATCH_BYTES = 4 * 1024 * 1024
mate_qkv_project = _lib.mate_qkv_project
mate_out_project = _lib.mate_out_project
mate_project_bwd_workspace_bytes = _lib.mate_project_bwd_workspace_bytes
mate_qkv_project_bwd = _lib.mate_qkv_project_bwd
mate_out_project_bwd = _lib.mate_out_project_bwd


def mate_status_string(status: int) -> str:
    return _lib.mate_status_string(int(status)).decode()


class MateError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {mate_status_string(status)} ({status})")
        self.status = status


def _check(status: int, where: str):
    if status != MATE_OK:
        raise MateError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MATE_F32
    if t.dtype == torch.bfloat16:
        return MATE_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t: torch.Tensor, name: str) -> int:
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous device tensor")
    return t.data_ptr()


@dataclass
class Segments:
    """Device buffer holding the tables of mate_build_segments for (B, N)."""
    buf: torch.Tensor
    B: int
    N: int


def build_segments(row_ids: torch.Tensor, col_ids: torch.Tensor, flags: torch.Tensor,
                   out: Segments | None = None, bucketed=None) -> Segments:
    """bucketed = (global_length, radius) builds the tables of the bucketed mode."""
    B, N = flags.shape
    assert row_ids.dtype == torch.int32 and col_ids.dtype == torch.int32 and flags.dtype == torch.uint8
    assert row_ids.shape == (B, N) and col_ids.shape == (B, N)
    nbytes = mate_segments_bytes(B, N)
    if nbytes == 0:
        raise MateError(MATE_ERR_SHAPE, "mate_segments_bytes")
    if out is None:
        out = Segments(torch.empty(nbytes, dtype=torch.uint8, device=flags.device), B, N)
    if bucketed is None:
        _check(mate_build_segments(_dev(row_ids, "row_ids"), _dev(col_ids, "col_ids"),
                                   _dev(flags, "flags"), B, N, out.buf.data_ptr(), _stream()),
               "mate_build_segments")
    else:
        _check(mate_build_segments_bucketed(_dev(row_ids, "row_ids"), _dev(col_ids, "col_ids"),
                                            _dev(flags, "flags"), B, N, int(bucketed[0]),
                                            int(bucketed[1]), out.buf.data_ptr(), _stream()),
               "mate_build_segments_bucketed")
    return out


def cell_positions(row_ids: torch.Tensor, col_ids: torch.Tensor, flags: torch.Tensor,
                   out: torch.Tensor | None = None) -> torch.Tensor:
    B, N = flags.shape
    assert row_ids.dtype == torch.int32 and col_ids.dtype == torch.int32 and flags.dtype == torch.uint8
    assert row_ids.shape == (B, N) and col_ids.shape == (B, N)
    if out is None:
        out = torch.empty((B, N), dtype=torch.int32, device=flags.device)
    assert out.dtype == torch.int32 and out.shape == (B, N)
    _check(mate_cell_positions(_dev(row_ids, "row_ids"), _dev(col_ids, "col_ids"), _dev(flags, "flags"),
                               B, N, _dev(out, "positions"), _stream()), "mate_cell_positions")
    return out


def segments_export(seg: Segments, view: int) -> dict:
    B, N = seg.B, seg.N
    perm = np.empty((B, N), np.int32)
    seg_off = np.empty((B, N + 1), np.int32)
    seg_of_tok = np.empty((B, N), np.int32)
    global_idx = np.empty((B, N), np.int32)
    counts = np.empty((B, 3), np.int32)
    _check(mate_segments_export(seg.buf.data_ptr(), B, N, view, perm.ctypes.data,
                                seg_off.ctypes.data, seg_of_tok.ctypes.data,
                                global_idx.ctypes.data, counts.ctypes.data, _stream()),
           "mate_segments_export")
    window = np.empty((B, N, 2), np.int32)
    _check(mate_segments_export_windows(seg.buf.data_ptr(), B, N, view, window.ctypes.data, _stream()),
           "mate_segments_export_windows")
    return dict(perm=perm, seg_off=seg_off, seg_of_tok=seg_of_tok, global_idx=global_idx,
                counts=counts, window=window)


def _head_kind_host(head_kind, H: int):
    hk = np.ascontiguousarray(np.asarray(head_kind, dtype=np.uint8))
    assert hk.shape == (H,)
    return hk


def workspace(B, H, N, D, dtype_code, for_bwd, device) -> torch.Tensor:
    n = mate_workspace_bytes(B, H, N, D, dtype_code, int(for_bwd))
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def _check_tables(seg: Segments, B: int, N: int):
    if (seg.B, seg.N) != (B, N) or seg.buf.numel() < mate_segments_bytes(B, N):
        raise MateError(MATE_ERR_SHAPE, f"segment tables are for (B, N) = ({seg.B}, {seg.N}), tensors for ({B}, {N})")


def attn_fwd(q, k, v, seg: Segments, head_kind, scale: float, out=None, lse=None, ws=None):
    B, H, N, D = q.shape
    _check_tables(seg, B, N)
    hk = _head_kind_host(head_kind, H)
    code = _dtype_code(q)
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    if ws is None:
        ws = workspace(B, H, N, D, code, False, q.device)
    _check(mate_attn_fwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), seg.buf.data_ptr(),
                         hk.ctypes.data, B, H, N, D, code, float(scale), _dev(out, "out"),
                         _dev(lse, "lse"), ws.data_ptr(), ws.numel(), _stream()),
           "mate_attn_fwd")
    return out, lse


def attn_bwd(q, k, v, out, lse, dout, seg: Segments, head_kind, scale: float,
             dq=None, dk=None, dv=None, ws=None):
    B, H, N, D = q.shape
    _check_tables(seg, B, N)
    hk = _head_kind_host(head_kind, H)
    code = _dtype_code(q)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(q) if dk is None else dk
    dv = torch.empty_like(q) if dv is None else dv
    if ws is None:
        ws = workspace(B, H, N, D, code, True, q.device)
    _check(mate_attn_bwd(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"),
                         _dev(lse, "lse"), _dev(dout, "dout"), seg.buf.data_ptr(),
                         hk.ctypes.data, B, H, N, D, code, float(scale), _dev(dq, "dq"),
                         _dev(dk, "dk"), _dev(dv, "dv"), ws.data_ptr(), ws.numel(), _stream()),
           "mate_attn_bwd")
    return dq, dk, dv


def attn_fwd_dense(q, k, v, row_ids, col_ids, flags, head_kind, scale: float, out=None, lse=None):
    """Dense-mask variant (no segment tables); bf16, N <= MATE_DENSE_MAX_N."""
    B, H, N, D = q.shape
    hk = _head_kind_host(head_kind, H)
    code = _dtype_code(q)
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    _check(mate_attn_fwd_dense(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(row_ids, "row_ids"),
                               _dev(col_ids, "col_ids"), _dev(flags, "flags"), hk.ctypes.data,
                               B, H, N, D, code, float(scale), _dev(out, "out"), _dev(lse, "lse"),
                               _stream()), "mate_attn_fwd_dense")
    return out, lse


def attn_bwd_dense(q, k, v, out, lse, dout, row_ids, col_ids, flags, head_kind, scale: float,
                   dq=None, dk=None, dv=None, ws=None):
    B, H, N, D = q.shape
    hk = _head_kind_host(head_kind, H)
    code = _dtype_code(q)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(q) if dk is None else dk
    dv = torch.empty_like(q) if dv is None else dv
    if ws is None:
        ws = torch.empty(max(mate_dense_workspace_bytes(B, H, N), 16), dtype=torch.uint8, device=q.device)
    _check(mate_attn_bwd_dense(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(out, "out"),
                               _dev(lse, "lse"), _dev(dout, "dout"), _dev(row_ids, "row_ids"),
                               _dev(col_ids, "col_ids"), _dev(flags, "flags"), hk.ctypes.data,
                               B, H, N, D, code, float(scale), _dev(dq, "dq"), _dev(dk, "dk"),
                               _dev(dv, "dv"), ws.data_ptr(), ws.numel(), _stream()),
           "mate_attn_bwd_dense")
    return dq, dk, dv


def qkv_project(x, w_qkv, bias, flags, H: int, q=None, k=None, v=None):
    """x [B,N,E] bf16, w_qkv [3*H*64, E] bf16, bias [3*H*64] float32 or None -> q, k, v [B,H,N,64]."""
    B, N, E = x.shape
    assert x.dtype == torch.bfloat16 and w_qkv.dtype == torch.bfloat16 and w_qkv.shape == (3 * H * 64, E)
    assert flags.dtype == torch.uint8 and flags.shape == (B, N)
    assert bias is None or (bias.dtype == torch.float32 and bias.shape == (3 * H * 64,))
    outs = [t if t is not None else torch.empty((B, H, N, 64), dtype=x.dtype, device=x.device) for t in (q, k, v)]
    for t in outs:
        assert t.dtype == x.dtype and t.shape == (B, H, N, 64)
    _check(mate_qkv_project(_dev(x, "x"), _dev(w_qkv, "w_qkv"), _dev(bias, "bias") if bias is not None else None,
                            _dev(flags, "flags"), B, N, H, E, MATE_BF16, *(_dev(t, "out") for t in outs),
                            _stream()), "mate_qkv_project")
    return tuple(outs)


def out_project(o, w_o, bias, flags, y=None):
    """o [B,H,N,64] bf16, w_o [E, H*64] bf16, bias [E] float32 or None -> y [B,N,E]."""
    B, H, N, D = o.shape
    E = w_o.shape[0]
    assert o.dtype == torch.bfloat16 and w_o.dtype == torch.bfloat16 and w_o.shape == (E, H * 64) and D == 64
    assert flags.dtype == torch.uint8 and flags.shape == (B, N)
    assert bias is None or (bias.dtype == torch.float32 and bias.shape == (E,))
    if y is None:
        y = torch.empty((B, N, E), dtype=o.dtype, device=o.device)
    assert y.dtype == o.dtype and y.shape == (B, N, E)
    _check(mate_out_project(_dev(o, "o"), _dev(w_o, "w_o"), _dev(bias, "bias") if bias is not None else None,
                            _dev(flags, "flags"), B, N, H, E, MATE_BF16, _dev(y, "y"), _stream()),
           "mate_out_project")
    return y


def _opt(t, name):
    return _dev(t, name) if t is not None else None


def project_bwd_workspace(B, N, H, E, device) -> torch.Tensor:
    n = mate_project_bwd_workspace_bytes(B, N, H, E)
    if n == 0:
        raise MateError(MATE_ERR_UNSUPPORTED, "mate_project_bwd_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def qkv_project_bwd(x, w_qkv, flags, dq, dk, dv, want_dx=True, want_dw=True, want_dbias=True, ws=None):
    """Gradients of qkv_project: dx [B,N,E] bf16, dw_qkv [3*H*64,E] float32, dbias [3*H*64] float32
    (None for the ones not wanted)."""
    B, N, E = x.shape
    H = dq.shape[1]
    assert x.dtype == torch.bfloat16 and w_qkv.shape == (3 * H * 64, E) and dq.shape == (B, H, N, 64)
    assert dk.shape == dq.shape and dv.shape == dq.shape and flags.shape == (B, N)
    dx = torch.empty_like(x) if want_dx else None
    dw = torch.empty((3 * H * 64, E), dtype=torch.float32, device=x.device) if want_dw else None
    db = torch.empty(3 * H * 64, dtype=torch.float32, device=x.device) if want_dbias else None
    ws = project_bwd_workspace(B, N, H, E, x.device) if ws is None else ws
    _check(mate_qkv_project_bwd(_dev(x, "x"), _dev(w_qkv, "w_qkv"), _dev(flags, "flags"), _dev(dq, "dq"),
                                _dev(dk, "dk"), _dev(dv, "dv"), B, N, H, E, MATE_BF16, _opt(dx, "dx"),
                                _opt(dw, "dw"), _opt(db, "dbias"), ws.data_ptr(), ws.numel(), _stream()),
           "mate_qkv_project_bwd")
    return dx, dw, db


def out_project_bwd(o, w_o, flags, dy, want_do=True, want_dw=True, want_dbias=True, ws=None):
    """Gradients of out_project: d_o [B,H,N,64] bf16, dw_o [E,H*64] float32, dbias [E] float32."""
    B, H, N, D = o.shape
    E = w_o.shape[0]
    assert o.dtype == torch.bfloat16 and w_o.shape == (E, H * 64) and dy.shape == (B, N, E) and D == 64
    d_o = torch.empty_like(o) if want_do else None
    dw = torch.empty((E, H * 64), dtype=torch.float32, device=o.device) if want_dw else None
    db = torch.empty(E, dtype=torch.float32, device=o.device) if want_dbias else None
    ws = project_bwd_workspace(B, N, H, E, o.device) if ws is None else ws
    _check(mate_out_project_bwd(_dev(o, "o"), _dev(w_o, "w_o"), _dev(flags, "flags"), _dev(dy, "dy"),
                                B, N, H, E, MATE_BF16, _opt(d_o, "d_o"), _opt(dw, "dw"), _opt(db, "dbias"),
                                ws.data_ptr(), ws.numel(), _stream()), "mate_out_project_bwd")
    return d_o, dw, db


def prefer_dense(B: int, H: int, N: int, dtype: torch.dtype = torch.bfloat16) -> bool:
    """Which of the two equivalent implementations to call (the library's own choice,
    mate_attn_prefers_dense: the measured break-even on MI355X)."""
    code = MATE_BF16 if dtype == torch.bfloat16 else MATE_F32
    return bool(mate_attn_prefers_dense(int(B), int(H), int(N), code))


def segments_status(seg: Segments) -> int:
    """MATE_OK, MATE_ERR_SHAPE or MATE_ERR_BAD_ID for a table buffer (synchronises)."""
    return int(mate_segments_status(seg.buf.data_ptr(), seg.B, seg.N, _stream()))
