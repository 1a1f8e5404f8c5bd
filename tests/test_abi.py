"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the header declares, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2206_07882_amd import qrnnt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "qrnnt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qrnnt_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = qrnnt.load()
    names = declared_functions()
    assert "qrnnt_lstm_step" in names and "qrnnt_joint_fuse" in names and len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in qrnnt.h but not exported"
    assert sorted(qrnnt.EXPORTS) == names
    assert lib.qrnnt_abi_version() == 3


def test_pack_bytes_formula():
    assert qrnnt.pack_bytes(2560, 240, qrnnt.LAYOUT_TILED_GATES) == 160 * 2 * 1024
    assert qrnnt.pack_bytes(46, 256, qrnnt.LAYOUT_TILED) == 3 * 2 * 1024
    assert qrnnt.pack_bytes(5, 70, qrnnt.LAYOUT_ROWMAJOR) == 5 * 64
    assert qrnnt.pack_bytes(6, 64, qrnnt.LAYOUT_TILED_GATES) == 0     # rows not a multiple of 4
    assert qrnnt.pack_bytes(0, 64, qrnnt.LAYOUT_TILED) == 0
    assert qrnnt.pack_bytes(4, 64, 9) == 0


def _qmat(ptr=0x1000, rows=64, cols=64, layout=qrnnt.LAYOUT_TILED_GATES):
    return qrnnt.CQMat(ptr, 0x2000, rows, cols, layout)


def _lstm(**kw):
    d = dict(w_ih=_qmat(), w_hh=_qmat(), bias=0x3000, x=0.1, h=1 / 7, hi=7.0, I=64, H=16)
    d.update(kw)
    return qrnnt.CLstm(d["w_ih"], d["w_hh"], d["bias"], d["x"], d["h"], d["hi"], d["I"], d["H"])


def test_argument_validation_happens_before_any_launch():
    lib = qrnnt.load()
    P = C.c_void_p
    # pack
    assert lib.qrnnt_pack_int4(None, 0, 4, 16, 1, P(0x1000), None, None) == 1
    assert lib.qrnnt_pack_int4(P(0x1000), 1, 4, 16, 1, P(0x1000), None, None) == 1      # fp32 needs row_scale_out
    assert lib.qrnnt_pack_int4(P(0x1000), 0, 0, 16, 1, P(0x1000), None, None) == 2
    assert lib.qrnnt_pack_int4(P(0x1000), 0, 4, 16, 7, P(0x1000), None, None) == 6
    assert lib.qrnnt_pack_int4(P(0x1000), 0, 6, 16, 2, P(0x1000), None, None) == 2
    assert lib.qrnnt_pack_int4(P(0x1000), 0, 4, 16, 1, P(0x1001), None, None) == 3
    assert lib.qrnnt_pack_int4(P(0x1000), 5, 4, 16, 1, P(0x1000), None, None) == 4
    # quantize
    assert lib.qrnnt_quantize_act(None, C.c_int64(4), C.c_float(1.0), P(0x1000), None) == 1
    assert lib.qrnnt_quantize_act(P(0x1000), C.c_int64(0), C.c_float(1.0), P(0x1000), None) == 2
    assert lib.qrnnt_quantize_act(P(0x1000), C.c_int64(4), C.c_float(-1.0), P(0x1000), None) == 4
    # lstm step: wrong layout, hidden size not a multiple of 16, shape mismatch, aliasing
    args = lambda L, x=P(0x1000), hp=P(0x2000), hn=P(0x3000), N=4: (
        C.byref(L), x, None, N, None, hp, P(0x4000), N, None, N, hn, P(0x5000), None, None, None, None)
    good = _lstm(w_ih=_qmat(rows=64, cols=64), w_hh=_qmat(rows=64, cols=16))
    assert lib.qrnnt_lstm_step(*args(_lstm(w_ih=_qmat(layout=1)))) == 6
    assert lib.qrnnt_lstm_step(*args(_lstm(H=24, w_ih=_qmat(rows=96), w_hh=_qmat(rows=96, cols=24)))) == 2
    assert lib.qrnnt_lstm_step(*args(_lstm(w_hh=_qmat(rows=64, cols=32)))) == 2
    assert lib.qrnnt_lstm_step(*args(good, x=None)) == 1
    assert lib.qrnnt_lstm_step(*args(good, x=P(0x1004))) == 3
    assert lib.qrnnt_lstm_step(*args(good, hp=P(0x3000))) == 4
    assert lib.qrnnt_lstm_step(*args(good, N=0)) == 2
    # lstm layer: workspace too small
    need = lib.qrnnt_lstm_layer_workspace(C.byref(good), 10, 2)
    assert need >= 10 * 2 * 64 * 4
    la = lambda ws_bytes, ld=16, off=0: (C.byref(good), P(0x1000), 10, 2, 0, None, None, P(0x2000), ld, off, None,
                                         None, None, None, P(0x10000), C.c_size_t(ws_bytes), None)
    assert lib.qrnnt_lstm_layer(*la(need - 1)) == 5
    assert lib.qrnnt_lstm_layer(*la(need, ld=8)) == 2
    # linear / joint / beam
    w = _qmat(rows=46, cols=256, layout=1)
    assert lib.qrnnt_linear(C.byref(w), None, C.c_float(0.1), None, 4, 0, P(0x1000), None, None) == 1
    big = _qmat(rows=256, cols=256, layout=1)
    assert lib.qrnnt_linear(C.byref(big), None, C.c_float(0.1), P(0x1000), 4, 1, P(0x2000), None, None) == 7
    assert lib.qrnnt_linear(C.byref(_qmat(rows=46, cols=256, layout=2)), None, C.c_float(0.1), P(0x1000), 4, 0,
                            P(0x2000), None, None) == 6
    ja = lambda blank: (P(0x1000), 10, P(0x2000), P(0x3000), C.byref(w), None, C.c_float(1 / 7), C.c_float(7.0), None,
                        None, C.c_float(0.3), C.c_float(0.5), C.c_float(0.0), 4, blank, None, None, P(0x4000), None)
    assert lib.qrnnt_joint_fuse(*ja(46)) == 4
    assert lib.qrnnt_beam_step(P(0x1000), P(0x2000), 2, 65, 46, 0, 0, P(0x3000), P(0x4000), P(0x5000), None) == 7
    assert lib.qrnnt_beam_step(P(0x1000), None, 2, 16, 46, 0, 0, P(0x3000), P(0x4000), P(0x5000), None) == 1
    assert lib.qrnnt_status_str(5) == b"workspace too small"


def test_validation_of_the_8bit_and_search_entry_points():
    lib = qrnnt.load()
    P = C.c_void_p
    # 8-bit blobs take twice the bytes of 4-bit ones, layout rules are the same
    assert qrnnt.pack_bytes(2560, 352, qrnnt.LAYOUT_TILED_GATES, 8) == 160 * 3 * 2048
    assert qrnnt.pack_bytes(5, 70, qrnnt.LAYOUT_ROWMAJOR, 8) == 5 * 128
    assert qrnnt.pack_bytes(6, 64, qrnnt.LAYOUT_TILED_GATES, 8) == 0
    assert lib.qrnnt_pack_int8(None, 0, 4, 16, 1, P(0x1000), None, None) == 1
    assert lib.qrnnt_pack_int8(P(0x1000), 0, 4, 16, 1, P(0x1001), None, None) == 3
    assert lib.qrnnt_quantize_act8(None, C.c_int64(4), C.c_float(1.0), P(0x1000), None) == 1
    assert lib.qrnnt_quantize_act8(P(0x1000), C.c_int64(4), C.c_float(0.0), P(0x1000), None) == 4
    # a width other than 4 or 8 is refused; the single-step entry points refuse 8-bit layers
    bad = _qmat(rows=46, cols=256, layout=1); bad.bits = 5
    assert lib.qrnnt_linear(C.byref(bad), None, C.c_float(0.1), P(0x1000), 4, 0, P(0x2000), None, None) == 4
    w8 = _qmat(rows=64, cols=64); w8.bits = 8
    h8 = _qmat(rows=64, cols=16); h8.bits = 8
    args = lambda L: (C.byref(L), P(0x1000), None, 4, None, P(0x2000), P(0x4000), 4, None, 4, P(0x3000), P(0x5000),
                      None, None, None, None)
    assert lib.qrnnt_lstm_step(*args(_lstm(w_ih=w8, w_hh=h8))) == 7
    assert lib.qrnnt_lstm_step(*args(_lstm(w_ih=w8, w_hh=_qmat(rows=64, cols=16)))) == 4      # widths must agree
    # linear_quant: the consumer's width is 4 or 8
    w = _qmat(rows=48, cols=256, layout=1)
    lq = lambda bits, q=P(0x2000): (C.byref(w), None, C.c_float(0.1), P(0x1000), 4, C.c_float(7.0), bits, q, None)
    assert lib.qrnnt_linear_quant(*lq(6)) == 4
    assert lib.qrnnt_linear_quant(*lq(4, None)) == 1
    # listed step group: list and count are required and aligned; one list serves steps of equal N that agree
    # on the use of parent and x_row
    good = _lstm(w_ih=_qmat(rows=64, cols=64), w_hh=_qmat(rows=64, cols=16))
    def desc(N=8, parent=0x6000, x_row=0x7000):
        return qrnnt.CStepDesc(C.addressof(good), 0x1000, x_row, 46, parent, 0x2000, 0x4000, N, None, N, 0x3000, 0x5000,
                               None, None)
    two = lambda a, b: (qrnnt.CStepDesc * 2)(a, b)
    listed = lambda arr, lst=P(0x8000), cnt=P(0x9000): lib.qrnnt_lstm_step_group_listed(arr, 2, lst, cnt, None)
    assert listed(two(desc(), desc()), lst=None) == 1
    assert listed(two(desc(), desc()), cnt=None) == 1
    assert listed(two(desc(), desc()), lst=P(0x8008)) == 3
    assert listed(two(desc(), desc(N=16))) == 4
    assert listed(two(desc(), desc(parent=None))) == 4
    assert listed(two(desc(), desc(x_row=None))) == 4
    assert lib.qrnnt_lstm_step_group_listed(None, 2, P(0x8000), P(0x9000), None) == 1
    assert lib.qrnnt_lstm_step_group_listed(two(desc(), desc()), 4, P(0x8000), P(0x9000), None) == 4
    # searches: a NULL model or impossible sizes give a zero workspace
    assert lib.qrnnt_decode_alsd_workspace(None, 10, 2, 4, 5) == 0
    assert lib.qrnnt_decode_workspace(None, 10, 2, 4, 2) == 0


def test_validation_of_the_row_quantizer_static_layer_and_diagnostics():
    lib = qrnnt.load()
    P = C.c_void_p
    # activation pitch: the next multiple of 16 bytes; non-positive widths have none
    lib.qrnnt_act_pitch.restype = C.c_int32
    assert [lib.qrnnt_act_pitch(c) for c in (1, 10, 15, 16, 17, 240, 340, 1280)] == [16, 16, 16, 16, 32, 240, 352, 1280]
    assert lib.qrnnt_act_pitch(0) == 0 and lib.qrnnt_act_pitch(-3) == 0
    # row quantizer: pointers, shape (pitch >= width and a multiple of 16), scale and width, alignment
    qr = lambda x=P(0x1000), rows=4, cols=10, inv=1.0, bits=4, q=P(0x2000), ld=16: lib.qrnnt_quantize_act_rows(
        x, C.c_int64(rows), cols, C.c_float(inv), bits, q, ld, None)
    assert qr(x=None) == 1 and qr(q=None) == 1
    assert qr(rows=0) == 2 and qr(cols=0) == 2 and qr(cols=20) == 2 and qr(ld=24) == 2
    assert qr(inv=0.0) == 4 and qr(bits=5) == 4
    assert qr(x=P(0x1002)) == 3 and qr(q=P(0x2004)) == 3
    # the layer call on the library's own scratch array: same checks as qrnnt_lstm_layer, then the size limit
    good = _lstm(w_ih=_qmat(rows=64, cols=64), w_hh=_qmat(rows=64, cols=16))
    ls = lambda T=10, B=2, x=P(0x1000), ld=16: lib.qrnnt_lstm_layer_static(C.byref(good), x, T, B, 0, None, None,
                                                                           P(0x2000), ld, 0, None, None, None)
    assert ls(x=None) == 1 and ls(ld=8) == 2 and ls(T=0) == 2
    too_long = (qrnnt.STATIC_WORKSPACE_BYTES // (2 * 64 * 4)) + 1        # the int32 input projection alone exceeds the array
    assert lib.qrnnt_lstm_layer_workspace(C.byref(good), too_long, 2) > qrnnt.STATIC_WORKSPACE_BYTES
    assert ls(T=too_long) == 5
    # alignment-length synchronous search: unknown flag bits are refused before anything else is looked at
    assert lib.qrnnt_decode_alsd_ex(None, P(0x1000), 10, 2, 4, 5, 15, C.c_uint32(2), None, P(0x2000), P(0x3000), P(0x4000),
                                    P(0x10000), C.c_size_t(1 << 20), None) in (1, 4)
    # matrix-instruction diagnostics: names for every form, argument checks
    lib.qrnnt_diag_mfma_form_name.restype = C.c_char_p
    n = lib.qrnnt_diag_mfma_forms()
    names = [lib.qrnnt_diag_mfma_form_name(i).decode() for i in range(n)]
    assert n >= 6 and len(set(names)) == n and names[0].startswith("int8") and lib.qrnnt_diag_mfma_form_name(n) == b""
    tops = C.c_double(0.0)
    dr = lambda form=0, iters=100, sink=P(0x1000), out=C.byref(tops): lib.qrnnt_diag_mfma_rate(form, iters, sink, out, None)
    assert dr(sink=None) == 1 and dr(out=None) == 1
    assert dr(form=n) == 4 and dr(form=-1) == 4 and dr(iters=0) == 4 and dr(iters=(1 << 22) + 1) == 4
    assert dr(sink=P(0x1002)) == 3


def test_product_path_does_not_reference_the_oracle():
    """The GPU package must never import or call the test oracle."""
    pkg = os.path.join(ROOT, "paper_2206_07882_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "liboracle" not in text, f


def test_bench_refuses_more_than_one_gpu():
    """One GPU per box: the benchmark says so and exits before touching any device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
