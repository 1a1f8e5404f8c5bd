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
