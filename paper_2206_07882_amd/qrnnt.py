"""ctypes binding of libqrnnt.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (torch is used
for device memory and streams, nothing else), checks dtype/contiguity, passes
raw pointers across the C ABI and raises :class:`QrnntError` on a non-zero
status.  There is no fallback: if the library is not built, :func:`load`
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqrnnt.so")

LAYOUT_ROWMAJOR, LAYOUT_TILED, LAYOUT_TILED_GATES = 0, 1, 2
SRC_INT8_CODES, SRC_FP32 = 0, 1

_lib = None


class QrnntError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load().qrnnt_status_str(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


class CQMat(C.Structure):
    _fields_ = [("packed", C.c_void_p), ("row_scale", C.c_void_p), ("rows", C.c_int32), ("cols", C.c_int32),
                ("layout", C.c_int32), ("bits", C.c_int32)]


class CLstm(C.Structure):
    _fields_ = [("w_ih", CQMat), ("w_hh", CQMat), ("bias", C.c_void_p), ("x_scale", C.c_float),
                ("h_scale", C.c_float), ("h_inv_scale", C.c_float), ("input_size", C.c_int32),
                ("hidden_size", C.c_int32)]


MAX_LAYERS = 4


class CNet(C.Structure):
    _fields_ = [("embed_codes", C.c_void_p), ("n_layers", C.c_int32), ("layer", CLstm * MAX_LAYERS), ("out", CQMat),
                ("out_bias", C.c_void_p), ("out_a_scale", C.c_float), ("log_softmax", C.c_int32),
                ("mid", CQMat), ("mid_bias", C.c_void_p), ("mid_scale", C.c_float), ("mid_inv_scale", C.c_float)]


class CModel(C.Structure):
    _fields_ = [("pred", CNet), ("lm_src", CNet), ("lm_ext", CNet), ("use_src", C.c_int32), ("use_ext", C.c_int32),
                ("joint_out", CQMat), ("joint_bias", C.c_void_p), ("z_scale", C.c_float), ("z_inv_scale", C.c_float),
                ("lambda_src", C.c_float), ("lambda_ext", C.c_float), ("rho", C.c_float), ("V", C.c_int32),
                ("blank", C.c_int32)]


EXPORTS = ["qrnnt_status_str", "qrnnt_abi_version", "qrnnt_pack_int4_bytes", "qrnnt_pack_int4", "qrnnt_unpack_int4",
           "qrnnt_pack_int8_bytes", "qrnnt_pack_int8", "qrnnt_quantize_act8", "qrnnt_act_pitch", "qrnnt_quantize_act_rows",
           "qrnnt_quantize_act", "qrnnt_linear", "qrnnt_linear_quant", "qrnnt_lstm_step", "qrnnt_lstm_layer_workspace", "qrnnt_lstm_layer",
           "qrnnt_input_projection", "qrnnt_input_table", "qrnnt_lstm_step_group", "qrnnt_lstm_step_group_listed",
           "qrnnt_bilstm_layer_workspace", "qrnnt_bilstm_layer", "qrnnt_lstm_layer_static",
           "qrnnt_joint_fuse", "qrnnt_beam_step", "qrnnt_decode_workspace", "qrnnt_decode", "qrnnt_decode_ex",
           "qrnnt_decode_alsd_workspace", "qrnnt_decode_alsd", "qrnnt_decode_alsd_ex",
           "qrnnt_diag_mfma_forms", "qrnnt_diag_mfma_form_name", "qrnnt_diag_mfma_rate"]

DECODE_EARLY_STOP = 1


def load():
    """Loads the built library; raises if it is missing (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2206_07882_amd.build`")
        lib = C.CDLL(LIB_PATH)
        lib.qrnnt_status_str.restype = C.c_char_p
        lib.qrnnt_status_str.argtypes = [C.c_int]
        lib.qrnnt_abi_version.restype = C.c_uint32
        lib.qrnnt_pack_int4_bytes.restype = C.c_size_t
        lib.qrnnt_pack_int4_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        lib.qrnnt_pack_int8_bytes.restype = C.c_size_t
        lib.qrnnt_pack_int8_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        if lib.qrnnt_abi_version() != 3:
            raise RuntimeError(f"{LIB_PATH} has ABI version {lib.qrnnt_abi_version()}, this binding needs 3: rebuild")
        lib.qrnnt_lstm_layer_workspace.restype = C.c_size_t
        lib.qrnnt_lstm_layer_workspace.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        lib.qrnnt_bilstm_layer_workspace.restype = C.c_size_t
        lib.qrnnt_bilstm_layer_workspace.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32]
        lib.qrnnt_decode_workspace.restype = C.c_size_t
        lib.qrnnt_decode_workspace.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        lib.qrnnt_decode_alsd_workspace.restype = C.c_size_t
        lib.qrnnt_decode_alsd_workspace.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        lib.qrnnt_diag_mfma_form_name.restype = C.c_char_p
        lib.qrnnt_act_pitch.restype = C.c_int32
        _lib = lib
    return _lib


def _ptr(t: Optional[torch.Tensor], dtype=None):
    if t is None:
        return None
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != 0:
        raise QrnntError(status, where)


def pack_bytes(rows: int, cols: int, layout: int, bits: int = 4) -> int:
    fn = load().qrnnt_pack_int8_bytes if bits == 8 else load().qrnnt_pack_int4_bytes
    return int(fn(rows, cols, layout))


class QMat:
    """A packed INT4 (or INT8) matrix on the device plus its per-row scales."""

    def __init__(self, packed: torch.Tensor, row_scale: torch.Tensor, rows: int, cols: int, layout: int, bits: int = 4):
        self.packed, self.row_scale, self.rows, self.cols, self.layout = packed, row_scale, rows, cols, layout
        self.bits = int(bits)

    def c(self) -> CQMat:
        return CQMat(self.packed.data_ptr(), self.row_scale.data_ptr(), self.rows, self.cols, self.layout, self.bits)


def _pack(bits: int, src: torch.Tensor, layout: int, row_scale: Optional[torch.Tensor]) -> QMat:
    assert src.dim() == 2 and src.is_cuda
    rows, cols = src.shape
    name = "qrnnt_pack_int8" if bits == 8 else "qrnnt_pack_int4"
    fn = getattr(load(), name)
    nbytes = pack_bytes(rows, cols, layout, bits)
    if nbytes == 0:
        _check(2, name + "_bytes")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=src.device)
    if src.dtype == torch.float32:
        scale = torch.empty(rows, dtype=torch.float32, device=src.device)
        st = fn(_ptr(src), SRC_FP32, rows, cols, layout, _ptr(packed), _ptr(scale), _stream())
    elif src.dtype == torch.int8:
        scale = row_scale if row_scale is not None else torch.ones(rows, dtype=torch.float32, device=src.device)
        st = fn(_ptr(src), SRC_INT8_CODES, rows, cols, layout, _ptr(packed), None, _stream())
    else:
        raise TypeError("src must be float32 or int8")
    _check(st, name)
    return QMat(packed, scale, rows, cols, layout, bits)


def pack_int4(src: torch.Tensor, layout: int, row_scale: Optional[torch.Tensor] = None) -> QMat:
    """fp32 weights (quantized per row) or int8 codes (row_scale given by the caller) -> QMat."""
    return _pack(4, src, layout, row_scale)


def pack_int8(src: torch.Tensor, layout: int, row_scale: Optional[torch.Tensor] = None) -> QMat:
    """The same at 8 bits (Sec. 3.2: the encoder's first layer and the RNN-T's linear layers)."""
    return _pack(8, src, layout, row_scale)


def unpack_int4(m: QMat) -> torch.Tensor:
    out = torch.empty((m.rows, m.cols), dtype=torch.int8, device=m.packed.device)
    cm = m.c()
    _check(load().qrnnt_unpack_int4(C.byref(cm), _ptr(out), _stream()), "qrnnt_unpack_int4")
    return out


def quantize_act(x: torch.Tensor, inv_scale: float) -> torch.Tensor:
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(load().qrnnt_quantize_act(_ptr(x, torch.float32), C.c_int64(x.numel()), C.c_float(inv_scale), _ptr(q),
                                     _stream()), "qrnnt_quantize_act")
    return q


def quantize_act8(x: torch.Tensor, inv_scale: float) -> torch.Tensor:
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(load().qrnnt_quantize_act8(_ptr(x, torch.float32), C.c_int64(x.numel()), C.c_float(inv_scale), _ptr(q),
                                      _stream()), "qrnnt_quantize_act8")
    return q


def act_pitch(cols: int) -> int:
    return int(load().qrnnt_act_pitch(C.c_int32(cols)))


def quantize_act_rows(x: torch.Tensor, inv_scale: float, bits: int = 4) -> torch.Tensor:
    """fp32 [..., cols] -> codes [..., act_pitch(cols)] (pad bytes zero): the form every LSTM entry point reads."""
    cols = x.shape[-1]
    rows = x.numel() // cols
    ld = act_pitch(cols)
    q = torch.empty(tuple(x.shape[:-1]) + (ld,), dtype=torch.int8, device=x.device)
    _check(load().qrnnt_quantize_act_rows(_ptr(x, torch.float32), C.c_int64(rows), C.c_int32(cols), C.c_float(inv_scale),
                                          C.c_int32(bits), _ptr(q), C.c_int32(ld), _stream()), "qrnnt_quantize_act_rows")
    return q


def linear(w: QMat, bias: Optional[torch.Tensor], a_scale: float, a: torch.Tensor, log_softmax: bool = False,
           want_acc: bool = False):
    N = a.shape[0]
    y = torch.empty((N, w.rows), dtype=torch.float32, device=a.device)
    acc = torch.empty((N, w.rows), dtype=torch.int32, device=a.device) if want_acc else None
    cw = w.c()
    _check(load().qrnnt_linear(C.byref(cw), _ptr(bias, torch.float32), C.c_float(a_scale), _ptr(a, torch.int8),
                               C.c_int32(N), C.c_int32(1 if log_softmax else 0), _ptr(y), _ptr(acc), _stream()),
           "qrnnt_linear")
    return (y, acc) if want_acc else y


def linear_quant(w: QMat, bias: Optional[torch.Tensor], a_scale: float, a: torch.Tensor, inv_scale: float,
                 bits: int = 4) -> torch.Tensor:
    N = a.shape[0]
    q = torch.empty((N, w.rows), dtype=torch.int8, device=a.device)
    cw = w.c()
    _check(load().qrnnt_linear_quant(C.byref(cw), _ptr(bias, torch.float32), C.c_float(a_scale), _ptr(a, torch.int8),
                                     C.c_int32(N), C.c_float(inv_scale), C.c_int32(bits), _ptr(q, torch.int8), _stream()),
           "qrnnt_linear_quant")
    return q


class Lstm:
    """One LSTM layer-direction on the device (TILED_GATES weights, fp32 bias)."""

    def __init__(self, w_ih: QMat, w_hh: QMat, bias: torch.Tensor, x_scale: float, h_scale: float = 1.0 / 7.0,
                 h_inv_scale: float = 7.0):
        self.w_ih, self.w_hh, self.bias = w_ih, w_hh, bias
        self.I, self.H = w_ih.cols, w_hh.cols
        self.x_scale, self.h_scale, self.h_inv_scale = float(x_scale), float(h_scale), float(h_inv_scale)

    def c(self) -> CLstm:
        return CLstm(self.w_ih.c(), self.w_hh.c(), self.bias.data_ptr(), self.x_scale, self.h_scale,
                     self.h_inv_scale, self.I, self.H)


def lstm_step(L: Lstm, x_codes, h_prev, c_prev, N: Optional[int] = None, x_row=None, parent=None, active=None,
              debug: bool = False):
    dev = h_prev.device
    if N is None:
        N = x_row.shape[0] if x_row is not None else x_codes.shape[0]
    H = L.H
    h_next = torch.empty((N, H), dtype=torch.int8, device=dev)
    c_next = torch.empty((N, H), dtype=torch.float32, device=dev)
    accx = acch = gates = None
    if debug:
        accx = torch.zeros((N, 4 * H), dtype=torch.int32, device=dev)
        acch = torch.zeros((N, 4 * H), dtype=torch.int32, device=dev)
        gates = torch.zeros((N, 4 * H), dtype=torch.float32, device=dev)
    cl = L.c()
    st = load().qrnnt_lstm_step(C.byref(cl), _ptr(x_codes, torch.int8), _ptr(x_row, torch.int32),
                                C.c_int32(x_codes.shape[0]), _ptr(parent, torch.int32), _ptr(h_prev, torch.int8),
                                _ptr(c_prev, torch.float32), C.c_int32(h_prev.shape[0]), _ptr(active, torch.uint8),
                                C.c_int32(N), _ptr(h_next), _ptr(c_next), _ptr(accx), _ptr(acch), _ptr(gates), _stream())
    _check(st, "qrnnt_lstm_step")
    if debug:
        return h_next, c_next, dict(accx=accx, acch=acch, gates=gates)
    return h_next, c_next


def lstm_step_into(L: Lstm, x_codes, h_prev, c_prev, h_next, c_next, N: int, x_row=None, parent=None, active=None):
    """qrnnt_lstm_step with caller-provided outputs (no allocation)."""
    cl = L.c()
    st = load().qrnnt_lstm_step(C.byref(cl), _ptr(x_codes, torch.int8), _ptr(x_row, torch.int32),
                                C.c_int32(x_codes.shape[0]), _ptr(parent, torch.int32), _ptr(h_prev, torch.int8),
                                _ptr(c_prev, torch.float32), C.c_int32(h_prev.shape[0]), _ptr(active, torch.uint8),
                                C.c_int32(N), _ptr(h_next, torch.int8), _ptr(c_next, torch.float32), None, None, None,
                                _stream())
    _check(st, "qrnnt_lstm_step")


class CStepDesc(C.Structure):
    _fields_ = [("L", C.c_void_p), ("x_codes", C.c_void_p), ("x_row", C.c_void_p), ("n_x_rows", C.c_int32),
                ("parent", C.c_void_p), ("h_prev", C.c_void_p), ("c_prev", C.c_void_p), ("n_slots", C.c_int32),
                ("active", C.c_void_p), ("N", C.c_int32), ("h_next", C.c_void_p), ("c_next", C.c_void_p),
                ("gx", C.c_void_p), ("gx_table", C.c_void_p), ("dbg_accx", C.c_void_p), ("dbg_acch", C.c_void_p),
                ("dbg_gates", C.c_void_p)]


class StepGroup:
    """Prepared argument block for qrnnt_lstm_step_group (built once, launched many times)."""

    def __init__(self, steps):
        """steps: list of dicts with keys L, x_codes, h_prev, c_prev, h_next, c_next, N and optional x_row, parent,
        active, gx (the input projection of the rows of x_codes, see input_projection), gx_table (input_table) and the
        debug outputs dbg_accx / dbg_acch (int32 [N, 4H]) / dbg_gates (fp32 [N, 4H])."""
        self._keep = []
        self.n = len(steps)
        self.arr = (CStepDesc * self.n)()
        p = lambda t: None if t is None else t.data_ptr()
        for i, d in enumerate(steps):
            cl = d["L"].c()
            self._keep.append((cl, d))
            self.arr[i] = CStepDesc(C.addressof(cl), p(d["x_codes"]), p(d.get("x_row")), d["x_codes"].shape[0],
                                    p(d.get("parent")), p(d["h_prev"]), p(d["c_prev"]), d["h_prev"].shape[0],
                                    p(d.get("active")), d["N"], p(d["h_next"]), p(d["c_next"]), p(d.get("gx")),
                                    p(d.get("gx_table")), p(d.get("dbg_accx")), p(d.get("dbg_acch")), p(d.get("dbg_gates")))

    def launch(self, list=None, n_list=None):
        """list [>= N, 4] int32 and n_list [1] int32 (device): only the listed hypotheses advance
        (qrnnt_lstm_step_group_listed)."""
        if list is None:
            _check(load().qrnnt_lstm_step_group(self.arr, C.c_int32(self.n), _stream()), "qrnnt_lstm_step_group")
        else:
            _check(load().qrnnt_lstm_step_group_listed(self.arr, C.c_int32(self.n), _ptr(list, torch.int32),
                                                       _ptr(n_list, torch.int32), _stream()),
                   "qrnnt_lstm_step_group_listed")


def input_projection(L: Lstm, x_codes: torch.Tensor, gx: Optional[torch.Tensor] = None, debug: bool = False):
    M = x_codes.shape[0]
    dev = x_codes.device
    if gx is None:
        gx = torch.empty((M, 4 * L.H), dtype=torch.int32, device=dev)
    acc = torch.zeros((M, 4 * L.H), dtype=torch.int32, device=dev) if debug else None
    cl = L.c()
    _check(load().qrnnt_input_projection(C.byref(cl), _ptr(x_codes, torch.int8), C.c_int32(M), _ptr(gx, torch.int32),
                                         _ptr(acc), _stream()), "qrnnt_input_projection")
    return gx, acc


def input_table(L: Lstm, gx: torch.Tensor) -> torch.Tensor:
    """fp32 form of an input projection with scales, bias and exp2 constants folded in (qrnnt_input_table)."""
    tab = torch.empty(gx.shape, dtype=torch.float32, device=gx.device)
    cl = L.c()
    _check(load().qrnnt_input_table(C.byref(cl), _ptr(gx, torch.int32), C.c_int32(gx.shape[0]), _ptr(tab), _stream()),
           "qrnnt_input_table")
    return tab


def lstm_layer_workspace(L: Lstm, T: int, B: int) -> int:
    cl = L.c()
    return int(load().qrnnt_lstm_layer_workspace(C.byref(cl), T, B))


def lstm_layer(L: Lstm, x_codes: torch.Tensor, reverse: bool = False, h0=None, c0=None, h_out=None, col_off: int = 0,
               want_last: bool = False, debug: bool = False, workspace: Optional[torch.Tensor] = None):
    T, B, I = x_codes.shape
    dev = x_codes.device
    H = L.H
    if h_out is None:
        h_out = torch.zeros((T, B, H), dtype=torch.int8, device=dev)
        col_off = 0
    ld = h_out.shape[2]
    need = lstm_layer_workspace(L, T, B)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    h_last = torch.empty((B, H), dtype=torch.int8, device=dev) if want_last else None
    c_last = torch.empty((B, H), dtype=torch.float32, device=dev) if want_last else None
    accx = torch.zeros((T, B, 4 * H), dtype=torch.int32, device=dev) if debug else None
    c_all = torch.zeros((T, B, H), dtype=torch.float32, device=dev) if debug else None
    cl = L.c()
    st = load().qrnnt_lstm_layer(C.byref(cl), _ptr(x_codes, torch.int8), C.c_int32(T), C.c_int32(B),
                                 C.c_int32(1 if reverse else 0), _ptr(h0, torch.int8), _ptr(c0, torch.float32),
                                 _ptr(h_out, torch.int8), C.c_int32(ld), C.c_int32(col_off), _ptr(h_last), _ptr(c_last),
                                 _ptr(accx), _ptr(c_all), _ptr(workspace), C.c_size_t(workspace.numel()), _stream())
    _check(st, "qrnnt_lstm_layer")
    return dict(h_out=h_out, h_last=h_last, c_last=c_last, accx=accx, c_all=c_all)


STATIC_WORKSPACE_BYTES = 32 << 20


def lstm_layer_static(L: Lstm, x_codes: torch.Tensor, h_out: torch.Tensor, reverse: bool = False, h0=None, c0=None,
                      col_off: int = 0, h_last=None, c_last=None):
    """qrnnt_lstm_layer_static: the layer with the library's own fixed workspace; every output is the caller's."""
    T, B, _ = x_codes.shape
    cl = L.c()
    st = load().qrnnt_lstm_layer_static(C.byref(cl), _ptr(x_codes, torch.int8), C.c_int32(T), C.c_int32(B),
                                        C.c_int32(1 if reverse else 0), _ptr(h0, torch.int8), _ptr(c0, torch.float32),
                                        _ptr(h_out, torch.int8), C.c_int32(h_out.shape[2]), C.c_int32(col_off),
                                        _ptr(h_last, torch.int8), _ptr(c_last, torch.float32), _stream())
    _check(st, "qrnnt_lstm_layer_static")
    return h_out


def bilstm_layer_workspace(fwd: Lstm, bwd: Lstm, T: int, B: int) -> int:
    cf, cb = fwd.c(), bwd.c()
    return int(load().qrnnt_bilstm_layer_workspace(C.byref(cf), C.byref(cb), T, B))


def bilstm_layer(fwd: Lstm, bwd: Lstm, x_codes: torch.Tensor, h_out: Optional[torch.Tensor] = None,
                 workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    T, B, _ = x_codes.shape
    dev = x_codes.device
    if h_out is None:
        h_out = torch.empty((T, B, 2 * fwd.H), dtype=torch.int8, device=dev)
    if workspace is None:
        workspace = torch.empty(bilstm_layer_workspace(fwd, bwd, T, B), dtype=torch.uint8, device=dev)
    cf, cb = fwd.c(), bwd.c()
    st = load().qrnnt_bilstm_layer(C.byref(cf), C.byref(cb), _ptr(x_codes, torch.int8), C.c_int32(T), C.c_int32(B),
                                   _ptr(h_out, torch.int8), _ptr(workspace), C.c_size_t(workspace.numel()), _stream())
    _check(st, "qrnnt_bilstm_layer")
    return h_out


def layer_error_flag(workspace: torch.Tensor, need: int) -> int:
    """The bounded-wait flag of the persistent recurrence (0 = all waits ended normally)."""
    return int(workspace[need - 256:need - 252].view(torch.int32).item())


def joint_fuse(enc_proj, frame_row, pred_proj, w_out: QMat, b_out, lp_src, lp_ext, lambda_src: float,
               lambda_ext: float, rho: float = 0.0, blank: int = 0, z_scale: float = 1.0 / 7.0,
               z_inv_scale: float = 7.0, want_lp: bool = False, want_zq: bool = False):
    N, J = pred_proj.shape
    V = w_out.rows
    dev = pred_proj.device
    enc2 = enc_proj.reshape(-1, J)
    fused = torch.empty((N, V), dtype=torch.float32, device=dev)
    lp = torch.empty((N, V), dtype=torch.float32, device=dev) if want_lp else None
    zq = torch.zeros((N, J), dtype=torch.int8, device=dev) if want_zq else None
    cw = w_out.c()
    st = load().qrnnt_joint_fuse(_ptr(enc2, torch.float32), C.c_int32(enc2.shape[0]), _ptr(frame_row, torch.int32),
                                 _ptr(pred_proj, torch.float32), C.byref(cw), _ptr(b_out, torch.float32),
                                 C.c_float(z_scale), C.c_float(z_inv_scale), _ptr(lp_src, torch.float32),
                                 _ptr(lp_ext, torch.float32), C.c_float(lambda_src), C.c_float(lambda_ext),
                                 C.c_float(rho), C.c_int32(N), C.c_int32(blank), _ptr(lp), _ptr(zq), _ptr(fused),
                                 _stream())
    _check(st, "qrnnt_joint_fuse")
    return fused, lp, zq


def beam_step(score: torch.Tensor, fused: torch.Tensor, blank: int = 0, force_blank: bool = False):
    B, W = score.shape
    V = fused.shape[-1]
    dev = score.device
    par = torch.empty((B, W), dtype=torch.int32, device=dev)
    tok = torch.empty((B, W), dtype=torch.int32, device=dev)
    ns = torch.empty((B, W), dtype=torch.float32, device=dev)
    st = load().qrnnt_beam_step(_ptr(score, torch.float32), _ptr(fused, torch.float32), C.c_int32(B), C.c_int32(W),
                                C.c_int32(V), C.c_int32(blank), C.c_int32(1 if force_blank else 0), _ptr(par),
                                _ptr(tok), _ptr(ns), _stream())
    _check(st, "qrnnt_beam_step")
    return par, tok, ns


class Net:
    """Prediction network or LM on the device: quantized embedding table,
    stacked LSTM layers, quantized output layer."""

    def __init__(self, embed_codes: torch.Tensor, layers, out: QMat, out_bias: Optional[torch.Tensor],
                 out_a_scale: float, log_softmax: bool, mid: Optional[QMat] = None,
                 mid_bias: Optional[torch.Tensor] = None, mid_scale: float = 0.0, mid_inv_scale: float = 0.0):
        self.embed_codes, self.layers, self.out, self.out_bias = embed_codes, list(layers), out, out_bias
        self.out_a_scale, self.log_softmax = float(out_a_scale), bool(log_softmax)
        self.mid, self.mid_bias, self.mid_scale, self.mid_inv_scale = mid, mid_bias, float(mid_scale), float(mid_inv_scale)

    def c(self) -> CNet:
        n = CNet()
        n.embed_codes = self.embed_codes.data_ptr()
        n.n_layers = len(self.layers)
        for i, l in enumerate(self.layers):
            n.layer[i] = l.c()
        n.out = self.out.c()
        n.out_bias = None if self.out_bias is None else self.out_bias.data_ptr()
        n.out_a_scale = self.out_a_scale
        n.log_softmax = 1 if self.log_softmax else 0
        if self.mid is not None:
            n.mid = self.mid.c()
            n.mid_bias = None if self.mid_bias is None else self.mid_bias.data_ptr()
            n.mid_scale, n.mid_inv_scale = self.mid_scale, self.mid_inv_scale
        return n


class Model:
    def __init__(self, pred: Net, lm_src: Optional[Net], lm_ext: Optional[Net], joint_out: QMat,
                 joint_bias: Optional[torch.Tensor], lambda_src: float, lambda_ext: float, rho: float = 0.0,
                 blank: int = 0, z_scale: float = 1.0 / 7.0, z_inv_scale: float = 7.0):
        self.pred, self.lm_src, self.lm_ext, self.joint_out, self.joint_bias = pred, lm_src, lm_ext, joint_out, joint_bias
        self.lambda_src, self.lambda_ext, self.rho = float(lambda_src), float(lambda_ext), float(rho)
        self.blank, self.z_scale, self.z_inv_scale = int(blank), float(z_scale), float(z_inv_scale)
        self.V, self.J = joint_out.rows, joint_out.cols

    def c(self) -> CModel:
        m = CModel()
        m.pred = self.pred.c()
        if self.lm_src is not None:
            m.lm_src = self.lm_src.c()
        if self.lm_ext is not None:
            m.lm_ext = self.lm_ext.c()
        m.use_src = 0 if self.lm_src is None else 1
        m.use_ext = 0 if self.lm_ext is None else 1
        m.joint_out = self.joint_out.c()
        m.joint_bias = None if self.joint_bias is None else self.joint_bias.data_ptr()
        m.z_scale, m.z_inv_scale = self.z_scale, self.z_inv_scale
        m.lambda_src, m.lambda_ext, m.rho = self.lambda_src, self.lambda_ext, self.rho
        m.V, m.blank = self.V, self.blank
        return m


def decode_workspace(model: Model, T: int, B: int, W: int, max_sym: int) -> int:
    cm = model.c()
    return int(load().qrnnt_decode_workspace(C.byref(cm), T, B, W, max_sym))


def decode(model: Model, enc_proj: torch.Tensor, W: int, max_sym: int, max_len: Optional[int] = None,
           workspace: Optional[torch.Tensor] = None, flags: int = 0):
    T, B, J = enc_proj.shape
    dev = enc_proj.device
    if max_len is None:
        max_len = max(1, T * max_sym)
    need = decode_workspace(model, T, B, W, max_sym)
    if need == 0:
        _check(2, "qrnnt_decode_workspace")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    tokens = torch.empty((B, W, max_len), dtype=torch.int32, device=dev)
    lens = torch.empty((B, W), dtype=torch.int32, device=dev)
    scores = torch.empty((B, W), dtype=torch.float32, device=dev)
    cm = model.c()
    st = load().qrnnt_decode_ex(C.byref(cm), _ptr(enc_proj, torch.float32), C.c_int32(T), C.c_int32(B), C.c_int32(W),
                                C.c_int32(max_sym), C.c_int32(max_len), C.c_uint32(flags), _ptr(tokens), _ptr(lens),
                                _ptr(scores), _ptr(workspace), C.c_size_t(workspace.numel()), _stream())
    _check(st, "qrnnt_decode_ex")
    return tokens, lens, scores


def decode_alsd_workspace(model: Model, T: int, B: int, W: int, u_max: int) -> int:
    cm = model.c()
    return int(load().qrnnt_decode_alsd_workspace(C.byref(cm), T, B, W, u_max))


ALSD_REUSE = 1


def decode_alsd(model: Model, enc_proj: torch.Tensor, W: int, u_max: int, max_len: Optional[int] = None,
                workspace: Optional[torch.Tensor] = None, flags: int = 0, stats: Optional[torch.Tensor] = None):
    """Alignment-length synchronous search with recombination; at most u_max labels per utterance.
    flags = ALSD_REUSE: label picks take over the states of a live hypothesis that holds their sequence;
    stats (int32 [2] on the device, zeroed by the caller) counts label picks and reuses."""
    T, B, J = enc_proj.shape
    dev = enc_proj.device
    if max_len is None:
        max_len = max(1, u_max)
    cm = model.c()
    need = int(load().qrnnt_decode_alsd_workspace(C.byref(cm), T, B, W, u_max))
    if need == 0:
        _check(2, "qrnnt_decode_alsd_workspace")
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    tokens = torch.empty((B, W, max_len), dtype=torch.int32, device=dev)
    lens = torch.empty((B, W), dtype=torch.int32, device=dev)
    scores = torch.empty((B, W), dtype=torch.float32, device=dev)
    st = load().qrnnt_decode_alsd_ex(C.byref(cm), _ptr(enc_proj, torch.float32), C.c_int32(T), C.c_int32(B), C.c_int32(W),
                                     C.c_int32(u_max), C.c_int32(max_len), C.c_uint32(flags), _ptr(stats, torch.int32),
                                     _ptr(tokens), _ptr(lens), _ptr(scores), _ptr(workspace),
                                     C.c_size_t(workspace.numel()), _stream())
    _check(st, "qrnnt_decode_alsd_ex")
    return tokens, lens, scores


def diag_mfma_rates(iters: int = 20000, device="cuda:0"):
    """[(name, TOP/s)] for every matrix-instruction form the library knows (qrnnt_diag_mfma_rate)."""
    lib = load()
    sink = torch.zeros(1, dtype=torch.float32, device=device)
    out = []
    for f in range(int(lib.qrnnt_diag_mfma_forms())):
        tops = C.c_double(0.0)
        _check(lib.qrnnt_diag_mfma_rate(C.c_int32(f), C.c_int32(iters), _ptr(sink), C.byref(tops), _stream()),
               "qrnnt_diag_mfma_rate")
        out.append((lib.qrnnt_diag_mfma_form_name(C.c_int32(f)).decode(), float(tops.value)))
    return out
