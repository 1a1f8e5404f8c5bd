"""Paths of the LSTM entry points that the measured configurations do not reach by themselves: the step-by-step
form of a layer (taken when the persistent recurrence cannot hold the layer), a given initial state on both forms,
input widths that are not a multiple of 16 (Sec. 2: 340 features, a small embedding), and the encoder's
surfacing of the recurrence's bounded-wait flag.  All against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from oracle import models as omodels
from paper_2206_07882_amd import synth
from tests.test_gpu_parity import _lstm_pair, assert_codes_close, assert_rel, dev, host, S_H, DEV, _tiled_gate_col

pytestmark = pytest.mark.gpu


def _padded(codes, fill):
    """[..., C] int8 -> [..., pitch(C)] with the padding bytes set to `fill` (they must not matter)."""
    C = codes.shape[-1]
    P = (C + 15) // 16 * 16
    out = np.full(codes.shape[:-1] + (P,), fill, np.int8)
    out[..., :C] = codes
    return out


def _teacher_forced_layer(L, x, hg, cg, reverse, h0, c0, what):
    T, B = x.shape[:2]
    order = range(T - 1, -1, -1) if reverse else range(T)
    hp = np.zeros((B, L.H), np.int8) if h0 is None else h0
    cp = np.zeros((B, L.H), np.float32) if c0 is None else c0
    for t in order:
        hr, cr, dbg = oracle.lstm_step(L, x[t], hp, cp, debug=True)
        assert_rel(cg[t], cr, f"{what} c t={t}")
        assert_codes_close(hg[t], hr, dbg["h_real"] * 7.0, f"{what} h t={t}")
        hp, cp = hg[t], cg[t]
    return hp, cp


@pytest.mark.parametrize("T,B,I,H,reverse,state", [(6, 3, 64, 1040, False, False), (5, 40, 64, 1040, True, True),
                                                   (4, 2, 32, 2048, False, True), (9, 5, 32, 64, False, True),
                                                   (7, 33, 240, 640, True, True), (30, 16, 16, 32, False, False),
                                                   (5, 112, 64, 640, True, True), (4, 130, 32, 1024, False, True)])
def test_lstm_layer_step_by_step_form_and_initial_state(gpu_lib, T, B, I, H, reverse, state):
    """H = 1040 and 2048 exceed what the persistent recurrence holds (H <= 1024), so the layer runs as one fused
    launch per time step (few utterances: the weight-streaming step kernel; 40: the tiled one, with a ragged
    row block since 1040 is not a multiple of 32); H = 64 and 640 take the persistent kernel, and so does H = 32, its
    smallest exchange (two workgroups per direction: the shape the benchmark times as the latency floor of a step).
    112 and 130 utterances make more workgroups of 16 cells than the device has compute units, so the persistent kernel
    runs in its form with 32 cells per workgroup (two row-tile groups per wave in the cell update).  Both forms with a
    given initial state (hidden codes and cell state), every step against one oracle step from the GPU's own
    previous state, final state returned."""
    q = gpu_lib
    s_x = float(np.float32(4) / np.float32(7))
    L, G = _lstm_pair(q, 1171 + I + H, I, H, s_x)
    x = synth.codes(1172 + T, (T, B, I), -8, 7)
    h0 = synth.codes(1173, (B, H), -7, 7) if state else None
    c0 = synth.normal(1174, (B, H), 0.6) if state else None
    need = q.lstm_layer_workspace(G, T, B)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = q.lstm_layer(G, dev(x), reverse=reverse, h0=None if h0 is None else dev(h0), c0=None if c0 is None else dev(c0),
                       want_last=True, debug=True, workspace=ws)
    if H <= 1024:
        assert q.layer_error_flag(ws, need) == 0
    hg, cg = host(out["h_out"]), host(out["c_all"])
    assert np.array_equal(host(out["accx"]).reshape(T * B, 4 * H), oracle.matmul_i32(L.w_ih, x.reshape(T * B, I)))
    hl, cl = _teacher_forced_layer(L, x, hg, cg, reverse, h0, c0, f"H={H}")
    assert np.array_equal(host(out["h_last"]), hl) and np.array_equal(host(out["c_last"]), cl)
    free, _, _, _ = oracle.lstm_layer(L, x, reverse=reverse, h0=h0, c0=c0)
    assert (free == hg).mean() >= 0.999
    if state:   # the state is used: from the zero state the first step's codes differ
        zero = host(q.lstm_layer(G, dev(x), reverse=reverse)["h_out"])
        t0 = T - 1 if reverse else 0
        assert not np.array_equal(zero[t0], hg[t0])


@pytest.mark.parametrize("I,H,N", [(340, 640, 32), (10, 768, 16), (15, 64, 48), (340, 640, 100), (10, 768, 1024),
                                   (130, 128, 7)])
def test_lstm_step_input_widths_that_are_not_a_multiple_of_16(gpu_lib, I, H, N):
    """Input rows of any width, stored with a pitch of the next multiple of 16; the padding bytes hold a non-zero
    code and must not reach the sums.  Few hypotheses: weight-streaming kernel; many: the tiled kernel's tail path."""
    q = gpu_lib
    s_x = float(np.float32(1.25) / np.float32(7))
    L, G = _lstm_pair(q, 1251 + I + H, I, H, s_x)
    assert q.act_pitch(I) == (I + 15) // 16 * 16 and q.act_pitch(16) == 16 and q.act_pitch(1) == 16
    x = synth.codes(1252 + N, (N, I), -8, 7)
    hp = synth.codes(1253 + N, (N, H), -7, 7)
    cp = synth.normal(1254 + N, (N, H), 0.7)
    hn, cn, dbg = q.lstm_step(G, dev(_padded(x, 7)), dev(hp), dev(cp), debug=True)
    hr, cr, dbg_r = oracle.lstm_step(L, x, hp, cp, debug=True)
    assert np.array_equal(host(dbg["accx"]), dbg_r["accx"]) and np.array_equal(host(dbg["acch"]), dbg_r["acch"])
    assert_rel(host(dbg["gates"]), dbg_r["gates"], "gates")
    assert_rel(host(cn), cr, "c")
    assert_codes_close(host(hn), hr, dbg_r["h_real"] * 7.0, "h codes")
    # the production build (no debug outputs) gives the same state
    hn2, cn2 = q.lstm_step(G, dev(_padded(x, -3)), dev(hp), dev(cp))
    assert torch.equal(hn, hn2) and torch.equal(cn, cn2)


@pytest.mark.parametrize("I,H,M", [(340, 640, 77), (10, 768, 46), (15, 2048, 46), (340, 640, 3000)])
def test_input_projection_and_quantizer_for_any_width(gpu_lib, I, H, M):
    """qrnnt_quantize_act_rows (fp32 rows of any width -> codes at the pitch the LSTM entry points read, padding
    zero) bit for bit against the oracle's quantizer, then the input projection of those rows."""
    q = gpu_lib
    L, G = _lstm_pair(q, 1371 + I, I, H, 0.1)
    xf = synth.normal(1372 + M, (M, I), 0.6)
    xf[0, :4] = np.array([0.5, 1.5, -2.5, 100.0], np.float32) * np.float32(4.0 / 7.0)      # ties and a clipped value
    inv = float(np.float32(7) / np.float32(4))
    codes = q.quantize_act_rows(dev(xf), inv)
    ref = oracle.quant_sym4(xf, inv)
    P = q.act_pitch(I)
    assert codes.shape == (M, P) and np.array_equal(host(codes)[:, :I], ref) and np.all(host(codes)[:, I:] == 0)
    c8 = q.quantize_act_rows(dev(xf), float(np.float32(127) / np.float32(4)), bits=8)
    assert np.array_equal(host(c8)[:, :I], oracle.quant_sym(xf, float(np.float32(127) / np.float32(4)), 8))
    gx, acc = q.input_projection(G, dev(_padded(ref, 5)), debug=True)
    want = oracle.matmul_i32(L.w_ih, ref)
    assert np.array_equal(host(acc), want)
    col = _tiled_gate_col(H)
    for g in range(4):
        assert np.array_equal(host(gx)[:, col[g]], want[:, g * H:(g + 1) * H])


def test_lstm_layer_340_features(gpu_lib):
    """A first encoder layer over 340 features (Sec. 2), both directions in one call, from fp32 features."""
    q = gpu_lib
    T, B, I, H = 7, 5, 340, 640
    s_x, inv_x = float(np.float32(4) / np.float32(7)), float(np.float32(7) / np.float32(4))
    Lf, Gf = _lstm_pair(q, 1471, I, H, s_x)
    Lb, Gb = _lstm_pair(q, 1481, I, H, s_x)
    feats = synth.normal(1472, (T, B, I), 1.0)
    xq = q.quantize_act_rows(dev(feats), inv_x)
    x = oracle.quant_sym4(feats, inv_x)
    need = q.bilstm_layer_workspace(Gf, Gb, T, B)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = host(q.bilstm_layer(Gf, Gb, xq, workspace=ws))
    assert q.layer_error_flag(ws, q.lstm_layer_workspace(Gf, T, B)) == 0 and q.layer_error_flag(ws, need) == 0
    for d, (L, order) in enumerate(((Lf, range(T)), (Lb, range(T - 1, -1, -1)))):
        hg = out[:, :, d * H:(d + 1) * H]
        hp = np.zeros((B, H), np.int8); cp = np.zeros((B, H), np.float32)
        for t in order:
            hr, cr, dbg = oracle.lstm_step(L, x[t], hp, cp, debug=True)
            assert_codes_close(hg[t], hr, dbg["h_real"] * 7.0, f"dir {d} h t={t}")
            hp, cp = hg[t], cr


def test_encoder_reports_the_recurrence_flag(gpu_lib):
    """Encoder.forward keeps the bounded-wait flag of every layer-direction (the workspace that holds it is reused
    by the next layer); check() raises on a non-zero one.  A normal run leaves all of them zero."""
    from paper_2206_07882_amd import model as gmodel
    m = synth.make_model(1, enc_layers=2)
    enc = gmodel.Encoder(m, DEV)
    feats = synth.features(1, 8, 3, m.feat_dim)
    enc._flags.fill_(7)                       # stale values must be overwritten by the forward
    enc.forward(dev(feats))
    assert enc._flags.cpu().tolist() == [0, 0, 0, 0]
    enc.check()
    enc._flags[2] = 1                         # what a timed-out wait in layer 1, forward direction, would leave
    with pytest.raises(RuntimeError):
        enc.check()


def test_matrix_instruction_diagnostics(gpu_lib):
    """qrnnt_diag_mfma_rate runs every form and reports plausible rates: positive, below twice the published fp6 / fp4
    peak, the int8 forms within reach of their 5.0 POP/s peak, and a chunk-shaped loop (LDS operand reads, barrier)
    never faster than the same instruction issued from registers alone."""
    rates = dict(gpu_lib.diag_mfma_rates(2000, DEV))
    assert len(rates) >= 9 and all(0.0 < t < 2.5e4 for t in rates.values()), rates
    for name in ("int8 16x16x64", "int8 32x32x32"):
        assert 2000.0 < rates[name] < 5500.0, rates
    for name, t in rates.items():
        if name.startswith("chunk loop"):
            base = name.split(": ", 1)[1]
            assert t <= 1.05 * rates[base], (name, t, rates[base])
