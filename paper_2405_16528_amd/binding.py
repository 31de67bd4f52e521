"""ctypes binding of libloqt.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used for device
memory and streams, nothing else), passes their pointers and pitches to the C ABI declared
in include/loqt.h and raises LoqtError on a non-zero status.  There is no CPU fallback: if
the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libloqt.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it with `python -m paper_2405_16528_amd.build` "
        "(there is no fallback path)")
lib = C.CDLL(_LIB_PATH)

F32, BF16 = 0, 1
OP_FWD, OP_BWD, OP_MERGE, OP_INIT, OP_FWD_RIGHT, OP_BWD_RIGHT, OP_MERGE_RIGHT = 0, 1, 2, 3, 4, 5, 6
OP_FWD_NQ, OP_BWD_NQ = 7, 8
OP_FWD_SAVE, OP_BWD_SAVED = 9, 10
PATH_AUTO, PATH_FUSED, PATH_PREPASS, PATH_FOLDED = 0, 1, 2, 3
TILE_AUTO, TILE_256x256, TILE_256x128, TILE_128x128 = 0, 1, 2, 3
STATUS_NAMES = {0: "LOQT_OK", 1: "LOQT_INVALID_ARG", 2: "LOQT_BAD_SHAPE", 3: "LOQT_MISALIGNED",
                4: "LOQT_WORKSPACE_TOO_SMALL", 5: "LOQT_LAUNCH_FAILED", 6: "LOQT_STATIC_SCRATCH_TOO_SMALL"}


class LoqtError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)}")


class NF4MatC(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("absmax", C.c_void_p), ("rows", C.c_int64),
                ("cols", C.c_int64), ("ld", C.c_int64)]


class MergeDescC(C.Structure):
    _fields_ = [("Wq", NF4MatC), ("codes_out", C.c_void_p), ("absmax_out", C.c_void_p),
                ("Pq", NF4MatC), ("B", C.c_void_p), ("ld_B", C.c_int64), ("s", C.c_float)]


_i64, _vp, _f, _i, _sz = C.c_int64, C.c_void_p, C.c_float, C.c_int, C.c_size_t
_P = C.POINTER
lib.loqt_status_string.restype = C.c_char_p
lib.loqt_status_string.argtypes = [_i]
lib.nf4_quantize.restype = _i
lib.nf4_quantize.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _i64, _vp]
lib.nf4_dequantize.restype = _i
lib.nf4_dequantize.argtypes = [_vp, _vp, _i64, _i64, _i64, _vp, _i, _i64, _vp]
lib.loqt_workspace_bytes.restype = _sz
lib.loqt_workspace_bytes.argtypes = [_i, _i64, _i64, _i64, _i64]
lib.loqt_linear_fwd.restype = _i
lib.loqt_linear_fwd.argtypes = [_vp, _i64, _i64, _P(NF4MatC), _P(NF4MatC), _vp, _i64, _f, _vp, _i64,
                                _vp, _sz, _vp]
lib.loqt_linear_bwd.restype = _i
lib.loqt_linear_bwd.argtypes = [_vp, _i64, _vp, _i64, _i64, _P(NF4MatC), _P(NF4MatC), _vp, _i64, _f,
                                _vp, _i64, _vp, _i, _i64, _i, _vp, _sz, _vp]
lib.loqt_linear_fwd_save.restype = _i
lib.loqt_linear_fwd_save.argtypes = [_vp, _i64, _i64, _P(NF4MatC), _P(NF4MatC), _vp, _i64, _f, _vp, _i64, _vp, _i64,
                                     _vp, _sz, _vp]
lib.loqt_linear_bwd_saved.restype = _i
lib.loqt_linear_bwd_saved.argtypes = [_vp, _i64, _vp, _i64, _i64, _P(NF4MatC), _i64, _f, _vp, _i64,
                                      _vp, _i64, _vp, _i, _i64, _i, _vp, _sz, _vp]
lib.loqt_merge_requant.restype = _i
lib.loqt_merge_requant.argtypes = [_P(NF4MatC), _vp, _vp, _P(NF4MatC), _vp, _i64, _f, _vp, _sz, _vp]
lib.loqt_merge_requant_batched.restype = _i
lib.loqt_merge_requant_batched.argtypes = [_i, _P(MergeDescC), _vp, _sz, _vp]
lib.loqt_merge_batched_workspace_bytes.restype = _sz
lib.loqt_merge_batched_workspace_bytes.argtypes = [_i, _P(MergeDescC)]
lib.loqt_linear_fwd_right.restype = _i
lib.loqt_linear_fwd_right.argtypes = lib.loqt_linear_fwd.argtypes
lib.loqt_linear_bwd_right.restype = _i
lib.loqt_linear_bwd_right.argtypes = lib.loqt_linear_bwd.argtypes
lib.loqt_merge_requant_right.restype = _i
lib.loqt_merge_requant_right.argtypes = lib.loqt_merge_requant.argtypes
lib.loqt_linear_fwd_nq.restype = _i
lib.loqt_linear_fwd_nq.argtypes = [_vp, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64, _i64, _f, _vp, _i64,
                                   _vp, _sz, _vp]
lib.loqt_linear_bwd_nq.restype = _i
lib.loqt_linear_bwd_nq.argtypes = [_vp, _i64, _vp, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64, _i64, _f,
                                   _vp, _i64, _vp, _i, _i64, _i, _vp, _sz, _vp]
lib.loqt_merge_nq.restype = _i
lib.loqt_merge_nq.argtypes = [_vp, _i64, _vp, _i64, _vp, _i64, _i64, _i64, _i64, _f, _vp]
lib.loqt_merge_dense.restype = _i
lib.loqt_merge_dense.argtypes = [_P(NF4MatC), _P(NF4MatC), _vp, _i64, _f, _vp, _i64, _vp, _sz, _vp]
lib.loqt_adam_step.restype = _i
lib.loqt_adam_step.argtypes = [_vp, _i64, _i64, _i64, _vp, _i, _i64, _vp, _vp, _i64, _f, _f, _f, _f, _i64, _vp]
lib.loqt_merge_schedule.restype = _i
lib.loqt_merge_schedule.argtypes = [C.c_double, C.c_double, _i64, _i, _P(_i64)]
lib.loqt_init_compensate.restype = _i
lib.loqt_init_compensate.argtypes = [_vp, _i64, _vp, _i64, _i64, _i64, _i64, _f, _i, _i, _vp, _vp, _i64, _vp, _i64,
                                     _vp, _sz, _vp]
lib.loqt_absmax_dq_workspace_bytes.restype = _sz
lib.loqt_absmax_dq_workspace_bytes.argtypes = [_i64]
lib.loqt_absmax_dq_compress.restype = _i
lib.loqt_absmax_dq_compress.argtypes = [_vp, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
lib.loqt_absmax_dq_static_max_n.restype = _i64
lib.loqt_absmax_dq_static_max_n.argtypes = []
lib.loqt_absmax_dq_compress_static.restype = _i
lib.loqt_absmax_dq_compress_static.argtypes = [_vp, _i64, _vp, _vp, _vp, _vp]
lib.loqt_absmax_dq_expand.restype = _i
lib.loqt_absmax_dq_expand.argtypes = [_vp, _vp, _vp, _i64, _vp, _vp]
lib.loqt_prepare.restype = _i
lib.loqt_prepare.argtypes = []
lib.loqt_set_path.restype = _i
lib.loqt_set_path.argtypes = [_i]
lib.loqt_plan_product.restype = _i
lib.loqt_plan_product.argtypes = [_i64, _i64, _i64, _P(_i64), _P(C.c_double)]
lib.loqt_set_tile.restype = _i
lib.loqt_set_tile.argtypes = [_i]
lib.loqt_resolved_path.restype = _i
lib.loqt_resolved_path.argtypes = [_i, _i64, _i64, _i64]
lib.loqt_timing_enable.restype = None
lib.loqt_timing_enable.argtypes = [_i]
lib.loqt_timing_slots.restype = _i
lib.loqt_timing_slots.argtypes = []
lib.loqt_timing_read.restype = _i
lib.loqt_timing_read.argtypes = [_i, _P(C.c_char_p), _P(_i64), _P(C.c_double)]


def _check(st: int, where: str) -> None:
    if st != 0:
        raise LoqtError(st, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _pitch(t: torch.Tensor) -> int:
    assert t.dim() == 2 and t.stride(1) == 1 and t.is_cuda
    return t.stride(0)


@dataclass
class NF4Tensor:
    """NF4 matrix on the device in the layout of include/loqt.h."""
    codes: torch.Tensor   # uint8 (rows, ld/2)
    absmax: torch.Tensor  # float32 (rows, ld/64)
    rows: int
    cols: int
    ld: int

    def c(self) -> NF4MatC:
        return NF4MatC(self.codes.data_ptr(), self.absmax.data_ptr(), self.rows, self.cols, self.ld)

    @staticmethod
    def empty(rows: int, cols: int, ld: Optional[int] = None, device="cuda") -> "NF4Tensor":
        ld = ld or (cols + 63) // 64 * 64
        return NF4Tensor(torch.empty((rows, ld // 2), dtype=torch.uint8, device=device),
                         torch.empty((rows, ld // 64), dtype=torch.float32, device=device), rows, cols, ld)


def nf4_quantize(w: torch.Tensor, out: Optional[NF4Tensor] = None, cols: Optional[int] = None) -> NF4Tensor:
    """w: float32 (rows, >=cols) on the GPU."""
    rows = w.shape[0]
    cols = cols if cols is not None else w.shape[1]
    out = out or NF4Tensor.empty(rows, cols, device=w.device)
    _check(lib.nf4_quantize(w.data_ptr(), rows, cols, _pitch(w), out.codes.data_ptr(), out.absmax.data_ptr(),
                            out.ld, _stream()), "nf4_quantize")
    return out


def nf4_dequantize(q: NF4Tensor, out: torch.Tensor) -> torch.Tensor:
    """out: float32 or bfloat16 (rows, >=cols) on the GPU; columns 0..cols-1 are written."""
    dt = {torch.float32: F32, torch.bfloat16: BF16}[out.dtype]
    _check(lib.nf4_dequantize(q.codes.data_ptr(), q.absmax.data_ptr(), q.rows, q.cols, q.ld, out.data_ptr(), dt,
                              _pitch(out), _stream()), "nf4_dequantize")
    return out


def loqt_workspace_bytes(op: int, T: int, out: int, inp: int, r: int) -> int:
    return int(lib.loqt_workspace_bytes(op, T, out, inp, r))


def loqt_linear_fwd(x, Wq: NF4Tensor, Pq: NF4Tensor, B, s: float, y, ws) -> torch.Tensor:
    T = x.shape[0]
    _check(lib.loqt_linear_fwd(x.data_ptr(), _pitch(x), T, C.byref(Wq.c()), C.byref(Pq.c()), B.data_ptr(),
                               _pitch(B), s, y.data_ptr(), _pitch(y), _ptr(ws), ws.numel() * ws.element_size(),
                               _stream()), "loqt_linear_fwd")
    return y


def loqt_linear_bwd(dy, x, Wq: NF4Tensor, Pq: NF4Tensor, B, s: float, dx, dB, accumulate: bool, ws):
    T = x.shape[0]
    dt = {torch.float32: F32, torch.bfloat16: BF16}[dB.dtype]
    _check(lib.loqt_linear_bwd(dy.data_ptr(), _pitch(dy), x.data_ptr(), _pitch(x), T, C.byref(Wq.c()),
                               C.byref(Pq.c()), B.data_ptr(), _pitch(B), s, _ptr(dx),
                               _pitch(dx) if dx is not None else 0, dB.data_ptr(), dt, _pitch(dB),
                               1 if accumulate else 0, _ptr(ws), ws.numel() * ws.element_size(), _stream()),
           "loqt_linear_bwd")
    return dx, dB


def loqt_linear_fwd_save(x, Wq: NF4Tensor, Pq: NF4Tensor, B, s: float, y, w_eff, ws) -> torch.Tensor:
    """Forward pass that also leaves the transient bf16 weight in w_eff (out, >= in) for loqt_linear_bwd_saved."""
    _check(lib.loqt_linear_fwd_save(x.data_ptr(), _pitch(x), x.shape[0], C.byref(Wq.c()), C.byref(Pq.c()),
                                    B.data_ptr(), _pitch(B), s, y.data_ptr(), _pitch(y), w_eff.data_ptr(),
                                    _pitch(w_eff), *_ws_args(ws), _stream()), "loqt_linear_fwd_save")
    return y


def loqt_linear_bwd_saved(dy, x, Pq: NF4Tensor, s: float, w_eff, dx, dB, accumulate: bool, ws):
    """Backward pass from the weight loqt_linear_fwd_save left behind; dx may be None."""
    dt = {torch.float32: F32, torch.bfloat16: BF16}[dB.dtype]
    _check(lib.loqt_linear_bwd_saved(dy.data_ptr(), _pitch(dy), x.data_ptr(), _pitch(x), x.shape[0], C.byref(Pq.c()),
                                     x.shape[1], s, w_eff.data_ptr(), _pitch(w_eff), _ptr(dx),
                                     _pitch(dx) if dx is not None else 0, dB.data_ptr(), dt, _pitch(dB),
                                     1 if accumulate else 0, *_ws_args(ws), _stream()), "loqt_linear_bwd_saved")
    return dx, dB


def workspace(op: int, T: int, out: int, inp: int, r: int, device="cuda") -> torch.Tensor:
    """A scratch buffer of loqt_workspace_bytes(...) bytes (torch's allocations are 256-byte aligned)."""
    return torch.empty(max(loqt_workspace_bytes(op, T, out, inp, r), 256), dtype=torch.uint8, device=device)


def _ws_args(ws):
    return (None, 0) if ws is None else (ws.data_ptr(), ws.numel() * ws.element_size())


def loqt_merge_requant(Wq: NF4Tensor, Pq: NF4Tensor, B, s: float, out: Optional[NF4Tensor] = None,
                       ws: Optional[torch.Tensor] = None) -> NF4Tensor:
    """out=None merges in place; ws=None allocates the workspace for this call."""
    out = out or Wq
    if ws is None:
        ws = workspace(OP_MERGE, 0, Wq.rows, Wq.cols, Pq.cols, Wq.codes.device)
    _check(lib.loqt_merge_requant(C.byref(Wq.c()), out.codes.data_ptr(), out.absmax.data_ptr(), C.byref(Pq.c()),
                                  B.data_ptr(), _pitch(B), s, *_ws_args(ws), _stream()), "loqt_merge_requant")
    return out


def make_merge_descs(layers):
    """layers: iterable of (Wq, out_or_None, Pq, B, s) -> ctypes array for the batched merge."""
    layers = list(layers)
    arr = (MergeDescC * len(layers))()
    for d, (Wq, out, Pq, B, s) in zip(arr, layers):
        out = out or Wq
        d.Wq, d.codes_out, d.absmax_out = Wq.c(), out.codes.data_ptr(), out.absmax.data_ptr()
        d.Pq, d.B, d.ld_B, d.s = Pq.c(), B.data_ptr(), _pitch(B), s
    return arr


def merge_descs_workspace_bytes(descs, full_groups: bool = True) -> int:
    """Workspace for loqt_merge_requant_batched: the size with which every group of layers is full (default), or
    the minimum (the largest single-layer need: groups of one layer)."""
    if full_groups:
        return max(int(lib.loqt_merge_batched_workspace_bytes(len(descs), descs)), 256)
    return max([loqt_workspace_bytes(OP_MERGE, 0, d.Wq.rows, d.Wq.cols, d.Pq.cols) for d in descs] + [256])


def loqt_merge_requant_batched(descs, ws: Optional[torch.Tensor] = None) -> None:
    if ws is None:
        ws = torch.empty(merge_descs_workspace_bytes(descs), dtype=torch.uint8, device="cuda")
    _check(lib.loqt_merge_requant_batched(len(descs), descs, *_ws_args(ws), _stream()), "loqt_merge_requant_batched")


def loqt_linear_fwd_right(x, Wq: NF4Tensor, Qq: NF4Tensor, Bp, s: float, y, ws) -> torch.Tensor:
    """Right-side variant: Wq (out, in), Qq (in, r), Bp bfloat16 (out, r)."""
    _check(lib.loqt_linear_fwd_right(x.data_ptr(), _pitch(x), x.shape[0], C.byref(Wq.c()), C.byref(Qq.c()),
                                     Bp.data_ptr(), _pitch(Bp), s, y.data_ptr(), _pitch(y), *_ws_args(ws),
                                     _stream()), "loqt_linear_fwd_right")
    return y


def loqt_linear_bwd_right(dy, x, Wq: NF4Tensor, Qq: NF4Tensor, Bp, s: float, dx, dBp, accumulate: bool, ws):
    """dx may be None; dBp float32 or bfloat16 (out, r)."""
    dt = {torch.float32: F32, torch.bfloat16: BF16}[dBp.dtype]
    _check(lib.loqt_linear_bwd_right(dy.data_ptr(), _pitch(dy), x.data_ptr(), _pitch(x), x.shape[0],
                                     C.byref(Wq.c()), C.byref(Qq.c()), Bp.data_ptr(), _pitch(Bp), s,
                                     _ptr(dx), _pitch(dx) if dx is not None else 0, dBp.data_ptr(), dt, _pitch(dBp),
                                     1 if accumulate else 0, *_ws_args(ws), _stream()), "loqt_linear_bwd_right")
    return dx, dBp


def loqt_merge_requant_right(Wq: NF4Tensor, Qq: NF4Tensor, Bp, s: float, out: Optional[NF4Tensor] = None,
                             ws: Optional[torch.Tensor] = None) -> NF4Tensor:
    out = out or Wq
    if ws is None:
        ws = workspace(OP_MERGE_RIGHT, 0, Wq.rows, Wq.cols, Qq.cols, Wq.codes.device)
    _check(lib.loqt_merge_requant_right(C.byref(Wq.c()), out.codes.data_ptr(), out.absmax.data_ptr(),
                                        C.byref(Qq.c()), Bp.data_ptr(), _pitch(Bp), s, *_ws_args(ws), _stream()),
           "loqt_merge_requant_right")
    return out


def loqt_linear_fwd_nq(x, W, P, B, s: float, y, ws) -> torch.Tensor:
    """LoQT-nq: W (out, in), P (out, r), B (r, in) bfloat16."""
    out, inp, r = W.shape[0], W.shape[1], P.shape[1]
    _check(lib.loqt_linear_fwd_nq(x.data_ptr(), _pitch(x), x.shape[0], W.data_ptr(), _pitch(W), P.data_ptr(), _pitch(P),
                                  B.data_ptr(), _pitch(B), out, inp, r, s, y.data_ptr(), _pitch(y), *_ws_args(ws),
                                  _stream()), "loqt_linear_fwd_nq")
    return y


def loqt_linear_bwd_nq(dy, x, W, P, B, s: float, dx, dB, accumulate: bool, ws):
    out, inp, r = W.shape[0], W.shape[1], P.shape[1]
    dt = {torch.float32: F32, torch.bfloat16: BF16}[dB.dtype]
    _check(lib.loqt_linear_bwd_nq(dy.data_ptr(), _pitch(dy), x.data_ptr(), _pitch(x), x.shape[0], W.data_ptr(),
                                  _pitch(W), P.data_ptr(), _pitch(P), B.data_ptr(), _pitch(B), out, inp, r, s,
                                  _ptr(dx), _pitch(dx) if dx is not None else 0, dB.data_ptr(), dt, _pitch(dB),
                                  1 if accumulate else 0, *_ws_args(ws), _stream()), "loqt_linear_bwd_nq")
    return dx, dB


def loqt_merge_nq(W, P, B, s: float) -> torch.Tensor:
    """W <- bf16(W + s P B) in place."""
    out, inp, r = W.shape[0], W.shape[1], P.shape[1]
    _check(lib.loqt_merge_nq(W.data_ptr(), _pitch(W), P.data_ptr(), _pitch(P), B.data_ptr(), _pitch(B), out, inp, r, s,
                             _stream()), "loqt_merge_nq")
    return W


def loqt_merge_dense(Wq: NF4Tensor, Pq: NF4Tensor, B, s: float, W_out: torch.Tensor,
                     ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """W_out: float32 (out, >= in): the unquantised merged weight deq(Wq) + s deq(Pq) B."""
    if ws is None:
        ws = workspace(OP_MERGE, 0, Wq.rows, Wq.cols, Pq.cols, Wq.codes.device)
    _check(lib.loqt_merge_dense(C.byref(Wq.c()), C.byref(Pq.c()), B.data_ptr(), _pitch(B), s, W_out.data_ptr(),
                                _pitch(W_out), *_ws_args(ws), _stream()), "loqt_merge_dense")
    return W_out


def loqt_adam_step(B: torch.Tensor, grad: torch.Tensor, m: torch.Tensor, v: torch.Tensor, lr: float, step: int,
                   beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
    """B bfloat16 (rows, cols) updated in place; grad float32 or bfloat16; m, v float32."""
    dt = {torch.float32: F32, torch.bfloat16: BF16}[grad.dtype]
    _check(lib.loqt_adam_step(B.data_ptr(), _pitch(B), B.shape[0], B.shape[1], grad.data_ptr(), dt, _pitch(grad),
                              m.data_ptr(), v.data_ptr(), _pitch(m), lr, beta1, beta2, eps, step, _stream()),
           "loqt_adam_step")


def loqt_absmax_dq_compress(absmax: torch.Tensor):
    """fp32 block scales (any shape, contiguous, taken flat) -> (codes uint8 [n], c1 float32 [ceil(n/256)],
    mean float32 [1]), all on the device."""
    a = absmax.reshape(-1)
    n = a.numel()
    dev = a.device
    codes = torch.empty(n, dtype=torch.uint8, device=dev)
    c1 = torch.empty((n + 255) // 256, dtype=torch.float32, device=dev)
    mean = torch.empty(1, dtype=torch.float32, device=dev)
    ws = torch.empty(max(int(lib.loqt_absmax_dq_workspace_bytes(n)), 8), dtype=torch.uint8, device=dev)
    _check(lib.loqt_absmax_dq_compress(a.data_ptr(), n, codes.data_ptr(), c1.data_ptr(), mean.data_ptr(),
                                       *_ws_args(ws), _stream()), "loqt_absmax_dq_compress")
    return codes, c1, mean


def loqt_absmax_dq_compress_static(absmax: torch.Tensor, codes: torch.Tensor, c1: torch.Tensor,
                                   mean: torch.Tensor) -> None:
    """The allocation-free variant: every output is the caller's (codes uint8 [n], c1 float32 [ceil(n/256)],
    mean float32 [1]); nothing is allocated here or in the library."""
    a = absmax.reshape(-1)
    _check(lib.loqt_absmax_dq_compress_static(a.data_ptr(), a.numel(), codes.data_ptr(), c1.data_ptr(),
                                              mean.data_ptr(), _stream()), "loqt_absmax_dq_compress_static")


def loqt_absmax_dq_expand(codes: torch.Tensor, c1: torch.Tensor, mean: torch.Tensor,
                          out: Optional[torch.Tensor] = None) -> torch.Tensor:
    n = codes.numel()
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=codes.device)
    _check(lib.loqt_absmax_dq_expand(codes.data_ptr(), c1.data_ptr(), mean.data_ptr(), n, out.data_ptr(), _stream()),
           "loqt_absmax_dq_expand")
    return out


def loqt_merge_schedule(n: int, tau: float = 100.0, psi: float = 1.2, cap: int = 2500):
    """The first n steps at which W is updated (host computation)."""
    arr = (_i64 * n)()
    _check(lib.loqt_merge_schedule(tau, psi, cap, n, arr), "loqt_merge_schedule")
    return list(arr)


def loqt_init_compensate(W: torch.Tensor, P: torch.Tensor, s: float, iters: int, B: torch.Tensor,
                         warm_start: bool = False, out: Optional[NF4Tensor] = None,
                         ws: Optional[torch.Tensor] = None) -> NF4Tensor:
    """W: float32 (out, in), P: float32 (out, r) with orthonormal columns, B: bfloat16 (r, in), in/out.
    Returns the quantised weight Q_c; B holds the matching factor."""
    o, i = W.shape
    r = P.shape[1]
    out = out or NF4Tensor.empty(o, i, device=W.device)
    if ws is None:
        ws = workspace(OP_INIT, 0, o, i, r, W.device)
    _check(lib.loqt_init_compensate(W.data_ptr(), _pitch(W), P.data_ptr(), _pitch(P), o, i, r, s, iters,
                                    1 if warm_start else 0, out.codes.data_ptr(), out.absmax.data_ptr(), out.ld,
                                    B.data_ptr(), _pitch(B), *_ws_args(ws), _stream()), "loqt_init_compensate")
    return out


def loqt_prepare() -> None:
    """Raise the LDS size of every kernel once (needed before a first call is recorded into a HIP graph)."""
    _check(lib.loqt_prepare(), "loqt_prepare")


def set_path(path: int) -> None:
    """PATH_AUTO, PATH_FUSED or PATH_PREPASS (process-wide)."""
    _check(lib.loqt_set_path(path), "loqt_set_path")


def plan_product(M: int, N: int, Nx: int = 0):
    """(columns that run on 256x256 tiles before a 128x128 tail launch, or 0; estimated rounds) -- host only."""
    n = _i64(0)
    c = C.c_double(0.0)
    _check(lib.loqt_plan_product(M, N, Nx, C.byref(n), C.byref(c)), "loqt_plan_product")
    return int(n.value), float(c.value)


def set_tile(tile: int) -> None:
    """TILE_AUTO, TILE_256x256, TILE_256x128 or TILE_128x128 (process-wide; tests and tuning)."""
    _check(lib.loqt_set_tile(tile), "loqt_set_tile")


def resolved_path(op: int, T: int, out: int, inp: int) -> int:
    return int(lib.loqt_resolved_path(op, T, out, inp))


def timing_enable(on: bool) -> None:
    lib.loqt_timing_enable(1 if on else 0)


def timing_read() -> dict:
    """{kernel name: (launches, total ms)} since the last timing_enable(True)."""
    out = {}
    for slot in range(lib.loqt_timing_slots()):
        name, n, ms = C.c_char_p(), _i64(), C.c_double()
        _check(lib.loqt_timing_read(slot, C.byref(name), C.byref(n), C.byref(ms)), "loqt_timing_read")
        out[name.value.decode()] = (n.value, ms.value)
    return out
