"""ctypes front end of the CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this package.  It loads ``oracle/liboracle.so`` (plain C, built with gcc by
:func:`build`) and wraps its functions for numpy arrays.  It holds no
arithmetic of its own and imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qrnnt_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
MAX_LAYERS = 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps every fp32
    product that decides a code a true fp32 product."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oq_quant_sym4.restype = C.c_int8
        _lib.oq_quant_sym4.argtypes = [C.c_float, C.c_float]
        _lib.oq_score_alignment.restype = C.c_float
        _lib.oq_tie_distance.restype = C.c_double
        _lib.oq_tie_distance.argtypes = [C.c_float, C.c_float, C.c_int]
        _lib.oq_struct_sizes.restype = C.c_int
        assert _lib.oq_struct_sizes(0) == C.sizeof(_CLstm)
        assert _lib.oq_struct_sizes(1) == C.sizeof(_CLinear)
        assert _lib.oq_struct_sizes(2) == C.sizeof(_CNet)
        assert _lib.oq_struct_sizes(3) == C.sizeof(_CModel)
    return _lib


def set_threads(n: int) -> None:
    omp = C.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def get_max_threads() -> int:
    omp = C.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def _p(a, ty=None):
    if a is None:
        return None
    return a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


class _CLstm(C.Structure):
    _fields_ = [("w_ih", C.c_void_p), ("w_hh", C.c_void_p), ("s_wih", C.c_void_p), ("s_whh", C.c_void_p),
                ("bias", C.c_void_p), ("I", C.c_int32), ("H", C.c_int32),
                ("s_x", C.c_float), ("s_h", C.c_float), ("inv_s_h", C.c_float), ("bits", C.c_int32)]


class _CLinear(C.Structure):
    _fields_ = [("w", C.c_void_p), ("s_w", C.c_void_p), ("bias", C.c_void_p),
                ("rows", C.c_int32), ("cols", C.c_int32), ("s_a", C.c_float), ("bits", C.c_int32)]


class _CNet(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("E", C.c_int32), ("L", C.c_int32), ("inv_s_e", C.c_float),
                ("layer", _CLstm * MAX_LAYERS), ("out", _CLinear), ("log_softmax", C.c_int32),
                ("has_mid", C.c_int32), ("mid", _CLinear), ("inv_s_mid", C.c_float)]


class _CModel(C.Structure):
    _fields_ = [("pred", _CNet), ("lm_src", _CNet), ("lm_ext", _CNet), ("joint_out", _CLinear),
                ("inv_s_z", C.c_float), ("lambda_src", C.c_float), ("lambda_ext", C.c_float), ("rho", C.c_float),
                ("V", C.c_int32), ("blank", C.c_int32), ("use_src", C.c_int32), ("use_ext", C.c_int32)]


# ---------------------------------------------------------------- quantizers

def quant_sym4(x, inv_s):
    x = _arr(x, np.float32)
    q = np.empty(x.shape, np.int8)
    lib().oq_quantize_sym4(_p(x), C.c_int64(x.size), C.c_float(inv_s), _p(q))
    return q


def quant_sym(x, inv_s, bits):
    """Symmetric b-bit codes clamp(rne(x * inv_s), -2^(b-1), 2^(b-1)-1) as int8."""
    x = _arr(x, np.float32)
    q = np.empty(x.shape, np.int8)
    lib().oq_quantize_sym(_p(x), C.c_int64(x.size), C.c_float(inv_s), C.c_int(bits), _p(q))
    return q


def tie_distance(x, inv_s, bits=4):
    """How close the quantizer's decision on x is to a rounding tie, in 4-bit code steps (inf where the clamp decides)."""
    return float(lib().oq_tie_distance(C.c_float(x), C.c_float(inv_s), C.c_int(bits)))


def quantize_asym(x, bits, a_lo, a_hi):
    x = _arr(x, np.float32)
    xi = np.empty(x.shape, np.int32)
    xq = np.empty(x.shape, np.float64)
    lib().oq_quantize_asym(_p(x), C.c_int64(x.size), C.c_int(bits), C.c_double(a_lo), C.c_double(a_hi), _p(xi), _p(xq))
    return xi, xq


def quantize_weight_rows(w, bits=4):
    w = _arr(w, np.float32)
    rows, cols = w.shape
    codes = np.empty((rows, cols), np.int8)
    scale = np.empty(rows, np.float32)
    if bits == 4:
        lib().oq_quantize_weight_rows(_p(w), C.c_int(rows), C.c_int(cols), _p(codes), _p(scale))
    else:
        lib().oq_quantize_weight_rows_bits(_p(w), C.c_int(rows), C.c_int(cols), C.c_int(bits), _p(codes), _p(scale))
    return codes, scale


def pack_rows(codes, cols_padded):
    codes = _arr(codes, np.int8)
    rows, cols = codes.shape
    out = np.empty((rows, cols_padded // 2), np.uint8)
    lib().oq_pack_rows(_p(codes), C.c_int(rows), C.c_int(cols), C.c_int(cols_padded), _p(out))
    return out


def unpack_rows(packed, cols):
    packed = _arr(packed, np.uint8)
    rows, bpr = packed.shape
    out = np.empty((rows, cols), np.int8)
    lib().oq_unpack_rows(_p(packed), C.c_int(rows), C.c_int(cols), C.c_int(bpr * 2), _p(out))
    return out


def matmul_i32(w, a):
    w = _arr(w, np.int8)
    a = _arr(a, np.int8)
    rows, K = w.shape
    N = a.shape[0]
    assert a.shape[1] == K
    acc = np.empty((N, rows), np.int32)
    lib().oq_matmul_i32(_p(w), C.c_int(rows), C.c_int(K), _p(a), C.c_int(N), _p(acc))
    return acc


# ---------------------------------------------------------------- layers

class Lstm:
    """One quantized LSTM layer-direction: integer codes + fp32 scales/bias."""

    def __init__(self, w_ih, s_wih, w_hh, s_whh, bias, s_x, s_h=1.0 / 7.0, inv_s_h=7.0, bits=4):
        self.bits = int(bits)
        self.w_ih = _arr(w_ih, np.int8)
        self.w_hh = _arr(w_hh, np.int8)
        self.s_wih = _arr(s_wih, np.float32)
        self.s_whh = _arr(s_whh, np.float32)
        self.bias = _arr(bias, np.float32)
        self.H = self.w_hh.shape[1]
        self.I = self.w_ih.shape[1]
        assert self.w_ih.shape[0] == 4 * self.H and self.w_hh.shape[0] == 4 * self.H
        self.s_x, self.s_h, self.inv_s_h = np.float32(s_x), np.float32(s_h), np.float32(inv_s_h)

    @classmethod
    def from_float(cls, w_ih, w_hh, bias, s_x, s_h=1.0 / 7.0, inv_s_h=7.0, bits=4):
        qi, si = quantize_weight_rows(w_ih, bits)
        qh, sh = quantize_weight_rows(w_hh, bits)
        return cls(qi, si, qh, sh, bias, s_x, s_h, inv_s_h, bits)

    def c(self):
        return _CLstm(_p(self.w_ih), _p(self.w_hh), _p(self.s_wih), _p(self.s_whh), _p(self.bias),
                      self.I, self.H, float(self.s_x), float(self.s_h), float(self.inv_s_h), self.bits)


class Linear:
    def __init__(self, w, s_w, bias, s_a, bits=4):
        self.bits = int(bits)
        self.w = _arr(w, np.int8)
        self.s_w = _arr(s_w, np.float32)
        self.bias = None if bias is None else _arr(bias, np.float32)
        self.rows, self.cols = self.w.shape
        self.s_a = np.float32(s_a)

    @classmethod
    def from_float(cls, w, bias, s_a, bits=4):
        q, s = quantize_weight_rows(w, bits)
        return cls(q, s, bias, s_a, bits)

    def c(self):
        return _CLinear(_p(self.w), _p(self.s_w), _p(self.bias), self.rows, self.cols, float(self.s_a), self.bits)


def lstm_step(L: Lstm, x, h_prev, c_prev, parent=None, active=None, debug=False):
    x = _arr(x, np.int8)
    h_prev = _arr(h_prev, np.int8)
    c_prev = _arr(c_prev, np.float32)
    N = x.shape[0]
    H = L.H
    parent_a = None if parent is None else _arr(parent, np.int32)
    active_a = None if active is None else _arr(active, np.uint8)
    h_next = np.empty((N, H), np.int8)
    c_next = np.empty((N, H), np.float32)
    accx = acch = gates = hreal = None
    if debug:
        accx = np.zeros((N, 4 * H), np.int32)
        acch = np.zeros((N, 4 * H), np.int32)
        gates = np.zeros((N, 4 * H), np.float64)
        hreal = np.zeros((N, H), np.float64)
    cl = L.c()
    lib().oq_lstm_step(C.byref(cl), _p(x), _p(parent_a), _p(h_prev), _p(c_prev), _p(active_a), C.c_int(N),
                       _p(h_next), _p(c_next), _p(accx), _p(acch), _p(gates), _p(hreal))
    if debug:
        return h_next, c_next, dict(accx=accx, acch=acch, gates=gates, h_real=hreal)
    return h_next, c_next


def lstm_layer(L: Lstm, x, reverse=False, h0=None, c0=None, h_out=None, col_off=0, want_c_all=False, utt_margin=None):
    """utt_margin: float64 [B], lowered in place to the smallest tie distance of each utterance's hidden-state
    quantizer decisions (oq_lstm_layer_margin)."""
    x = _arr(x, np.int8)
    T, B, I = x.shape
    assert I == L.I
    H = L.H
    if h_out is None:
        h_out = np.zeros((T, B, H), np.int8)
        col_off = 0
    assert h_out.dtype == np.int8 and h_out.flags.c_contiguous
    ld = h_out.shape[2]
    h_last = np.empty((B, H), np.int8)
    c_last = np.empty((B, H), np.float32)
    c_all = np.empty((T, B, H), np.float32) if want_c_all else None
    h0a = None if h0 is None else _arr(h0, np.int8)
    c0a = None if c0 is None else _arr(c0, np.float32)
    cl = L.c()
    if utt_margin is not None:
        assert utt_margin.dtype == np.float64 and utt_margin.shape == (B,) and utt_margin.flags.c_contiguous
        lib().oq_lstm_layer_margin(C.byref(cl), _p(x), C.c_int(T), C.c_int(B), C.c_int(1 if reverse else 0), _p(h0a),
                                   _p(c0a), _p(h_out), C.c_int(ld), C.c_int(col_off), _p(h_last), _p(c_last), _p(c_all),
                                   _p(utt_margin))
        return h_out, h_last, c_last, c_all
    lib().oq_lstm_layer(C.byref(cl), _p(x), C.c_int(T), C.c_int(B), C.c_int(1 if reverse else 0), _p(h0a), _p(c0a),
                        _p(h_out), C.c_int(ld), C.c_int(col_off), _p(h_last), _p(c_last), _p(c_all))
    return h_out, h_last, c_last, c_all


def linear(P: Linear, a, want_acc=False):
    a = _arr(a, np.int8)
    N = a.shape[0]
    y = np.empty((N, P.rows), np.float32)
    acc = np.empty((N, P.rows), np.int32) if want_acc else None
    cp = P.c()
    lib().oq_linear(C.byref(cp), _p(a), C.c_int(N), _p(y), _p(acc))
    return (y, acc) if want_acc else y


def log_softmax(x):
    x = _arr(x, np.float32)
    N, V = x.shape
    lp = np.empty((N, V), np.float32)
    lib().oq_log_softmax(_p(x), C.c_int(N), C.c_int(V), _p(lp))
    return lp


def joint_z(enc_proj, frame_row, pred_proj, inv_s_z=7.0, bits=4):
    enc_proj = _arr(enc_proj, np.float32)
    pred_proj = _arr(pred_proj, np.float32)
    frame_row = _arr(frame_row, np.int32)
    N, J = pred_proj.shape
    zq = np.empty((N, J), np.int8)
    zr = np.empty((N, J), np.float64)
    lib().oq_joint_z(_p(enc_proj), _p(frame_row), _p(pred_proj), C.c_int(N), C.c_int(J), C.c_float(inv_s_z), C.c_int(bits),
                     _p(zq), _p(zr))
    return zq, zr


def joint_out(out: Linear, zq, lp_src, lp_ext, lambda_src, lambda_ext, rho=0.0, blank=0):
    zq = _arr(zq, np.int8)
    N = zq.shape[0]
    V = out.rows
    ls = None if lp_src is None else _arr(lp_src, np.float32)
    le = None if lp_ext is None else _arr(lp_ext, np.float32)
    lp = np.empty((N, V), np.float32)
    fused = np.empty((N, V), np.float32)
    co = out.c()
    lib().oq_joint_out(C.byref(co), _p(zq), _p(ls), _p(le), C.c_float(lambda_src), C.c_float(lambda_ext), C.c_float(rho),
                       C.c_int(N), C.c_int(blank), _p(lp), _p(fused))
    return lp, fused


def joint_fuse(enc_proj, frame_row, pred_proj, out: Linear, lp_src, lp_ext, lambda_src, lambda_ext,
               rho=0.0, blank=0, inv_s_z=7.0):
    enc_proj = _arr(enc_proj, np.float32)
    pred_proj = _arr(pred_proj, np.float32)
    frame_row = _arr(frame_row, np.int32)
    N, J = pred_proj.shape
    V = out.rows
    ls = None if lp_src is None else _arr(lp_src, np.float32)
    le = None if lp_ext is None else _arr(lp_ext, np.float32)
    zq = np.empty((N, J), np.int8)
    lp = np.empty((N, V), np.float32)
    fused = np.empty((N, V), np.float32)
    co = out.c()
    lib().oq_joint_fuse(_p(enc_proj), _p(frame_row), _p(pred_proj), C.byref(co), C.c_float(inv_s_z), _p(ls), _p(le),
                        C.c_float(lambda_src), C.c_float(lambda_ext), C.c_float(rho), C.c_int(N), C.c_int(blank),
                        _p(zq), _p(lp), _p(fused))
    return zq, lp, fused


def beam_step(score, fused, blank=0, force_blank=False, want_gap=False):
    """want_gap: also returns, per utterance, the smallest difference between consecutive values among the picks and
    the best candidate left out (inf when nothing is ranked against anything)."""
    score = _arr(score, np.float32)
    fused = _arr(fused, np.float32)
    B, W = score.shape
    V = fused.shape[-1]
    assert fused.size == B * W * V
    par = np.empty((B, W), np.int32)
    tok = np.empty((B, W), np.int32)
    ns = np.empty((B, W), np.float32)
    if want_gap:
        gap = np.full(B, np.inf, np.float64)
        lib().oq_beam_step_gap(_p(score), _p(fused), C.c_int(B), C.c_int(W), C.c_int(V), C.c_int(blank),
                               C.c_int(1 if force_blank else 0), _p(par), _p(tok), _p(ns), _p(gap))
        return par, tok, ns, gap
    lib().oq_beam_step(_p(score), _p(fused), C.c_int(B), C.c_int(W), C.c_int(V), C.c_int(blank),
                       C.c_int(1 if force_blank else 0), _p(par), _p(tok), _p(ns))
    return par, tok, ns


# ---------------------------------------------------------------- networks

class Net:
    """Embedding -> quantizer -> stacked LSTM steps -> linear (-> log-softmax)."""

    def __init__(self, embed, alpha_e, layers, out: Linear, log_softmax: bool, mid: Linear = None, alpha_mid=None):
        """mid: optional bottleneck layer between the LSTM stack and out (Sec. 2, external LM); its
        output is quantized with boundary alpha_mid and out.s_a must be alpha_mid / 7."""
        self.mid = mid
        self.inv_s_mid = np.float32(0.0) if mid is None else np.float32(np.float32(7.0) / np.float32(alpha_mid))
        self.embed = _arr(embed, np.float32)
        self.E = self.embed.shape[1]
        self.inv_s_e = np.float32(np.float32(7.0) / np.float32(alpha_e))
        self.s_e = np.float32(np.float32(alpha_e) / np.float32(7.0))
        self.layers = list(layers)
        self.out = out
        self.log_softmax = bool(log_softmax)

    def c(self):
        n = _CNet()
        n.embed = _p(self.embed).value
        n.E = self.E
        n.L = len(self.layers)
        n.inv_s_e = float(self.inv_s_e)
        for i, l in enumerate(self.layers):
            n.layer[i] = l.c()
        n.out = self.out.c()
        n.log_softmax = 1 if self.log_softmax else 0
        n.has_mid = 0 if self.mid is None else 1
        if self.mid is not None:
            n.mid = self.mid.c()
            n.inv_s_mid = float(self.inv_s_mid)
        return n


def net_run(net: Net, tokens):
    tokens = _arr(tokens, np.int32)
    y = np.empty((tokens.size, net.out.rows), np.float32)
    cn = net.c()
    lib().oq_net_run(C.byref(cn), _p(tokens), C.c_int(tokens.size), _p(y))
    return y


class Model:
    def __init__(self, pred: Net, lm_src, lm_ext, joint_out_lin: Linear, lambda_src, lambda_ext, rho=0.0,
                 blank=0, inv_s_z=7.0):
        self.pred, self.lm_src, self.lm_ext, self.joint_out = pred, lm_src, lm_ext, joint_out_lin
        self.lambda_src, self.lambda_ext, self.rho = float(lambda_src), float(lambda_ext), float(rho)
        self.blank, self.inv_s_z = int(blank), float(inv_s_z)
        self.V = joint_out_lin.rows

    def c(self):
        m = _CModel()
        m.pred = self.pred.c()
        if self.lm_src is not None:
            m.lm_src = self.lm_src.c()
        if self.lm_ext is not None:
            m.lm_ext = self.lm_ext.c()
        m.joint_out = self.joint_out.c()
        m.inv_s_z = self.inv_s_z
        m.lambda_src, m.lambda_ext, m.rho = self.lambda_src, self.lambda_ext, self.rho
        m.V, m.blank = self.V, self.blank
        m.use_src = 0 if self.lm_src is None else 1
        m.use_ext = 0 if self.lm_ext is None else 1
        return m


def decode(model: Model, enc_proj, W, max_sym, max_len=None, margins=False):
    """margins: also returns (qmargin [B], smargin [B]) of oq_decode_margins: the smallest quantizer tie distance and
    the smallest selection gap met on each utterance's way."""
    enc_proj = _arr(enc_proj, np.float32)
    T, B, J = enc_proj.shape
    if max_len is None:
        max_len = T * max_sym
    tokens = np.empty((B, W, max_len), np.int32)
    lens = np.empty((B, W), np.int32)
    scores = np.empty((B, W), np.float32)
    cm = model.c()
    if margins:
        qm, sm = np.empty(B, np.float64), np.empty(B, np.float64)
        lib().oq_decode_margins(C.byref(cm), _p(enc_proj), C.c_int(T), C.c_int(B), C.c_int(W), C.c_int(max_sym),
                                C.c_int(max_len), _p(tokens), _p(lens), _p(scores), _p(qm), _p(sm))
        return tokens, lens, scores, qm, sm
    lib().oq_decode(C.byref(cm), _p(enc_proj), C.c_int(T), C.c_int(B), C.c_int(W), C.c_int(max_sym), C.c_int(max_len),
                    _p(tokens), _p(lens), _p(scores))
    return tokens, lens, scores


def decode_alsd(model: Model, enc_proj, W, u_max, max_len=None, margins=False):
    """Alignment-length synchronous search with recombination; at most u_max labels per utterance.
    margins: as in decode (oq_decode_alsd_margins)."""
    enc_proj = _arr(enc_proj, np.float32)
    T, B, J = enc_proj.shape
    if max_len is None:
        max_len = max(1, u_max)
    tokens = np.empty((B, W, max_len), np.int32)
    lens = np.empty((B, W), np.int32)
    scores = np.empty((B, W), np.float32)
    cm = model.c()
    if margins:
        qm, sm = np.empty(B, np.float64), np.empty(B, np.float64)
        lib().oq_decode_alsd_margins(C.byref(cm), _p(enc_proj), C.c_int(T), C.c_int(B), C.c_int(W), C.c_int(u_max),
                                     C.c_int(max_len), _p(tokens), _p(lens), _p(scores), _p(qm), _p(sm))
        return tokens, lens, scores, qm, sm
    lib().oq_decode_alsd(C.byref(cm), _p(enc_proj), C.c_int(T), C.c_int(B), C.c_int(W), C.c_int(u_max),
                         C.c_int(max_len), _p(tokens), _p(lens), _p(scores))
    return tokens, lens, scores


def decode_alsd_cached(model: Model, enc_proj, W, u_max, cache_mode, max_len=None):
    """oq_decode_alsd_cached: the search with reuse of cached hypotheses (cache_mode 0 none, 1 the current beam,
    2 every sequence ever extended).  Returns (tokens, lens, scores, requested [B], performed [B])."""
    enc_proj = _arr(enc_proj, np.float32)
    T, B, J = enc_proj.shape
    if max_len is None:
        max_len = max(1, u_max)
    tokens = np.empty((B, W, max_len), np.int32)
    lens = np.empty((B, W), np.int32)
    scores = np.empty((B, W), np.float32)
    req, done = np.zeros(B, np.int64), np.zeros(B, np.int64)
    cm = model.c()
    lib().oq_decode_alsd_cached(C.byref(cm), _p(enc_proj), C.c_int(T), C.c_int(B), C.c_int(W), C.c_int(u_max),
                                C.c_int(max_len), _p(tokens), _p(lens), _p(scores), C.c_int(cache_mode), _p(req), _p(done))
    return tokens, lens, scores, req, done


def score_alignment(model: Model, enc_proj, b, actions):
    enc_proj = _arr(enc_proj, np.float32)
    T, B, J = enc_proj.shape
    actions = _arr(actions, np.int32)
    cm = model.c()
    return float(lib().oq_score_alignment(C.byref(cm), _p(enc_proj), C.c_int(B), C.c_int(b), _p(actions),
                                          C.c_int(actions.size)))


def quant_calls_reset():
    lib().oq_quant_calls_reset()


def quant_calls():
    f = lib().oq_quant_calls_get
    f.restype = C.c_long
    return int(f())
