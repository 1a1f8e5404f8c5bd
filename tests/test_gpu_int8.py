"""Parity of the 8-bit paths (Sec. 3.2: the first encoder layer and the RNN-T's linear layers stay at 8 bits)
with the CPU oracle, through the C ABI.  Same bars as the 4-bit tests: packed bytes, weight codes and int32
sums bit-exact; fp32 values within 1e-5 relative; requantised codes equal except at rounding ties."""
import numpy as np
import pytest
import torch

import oracle
from oracle import models as omodels
from paper_2206_07882_amd import synth

from .test_gpu_parity import assert_codes_close, assert_rel, dev, host, _tiled_gate_col, DEV
from .test_gpu_decode import _compare_beams

pytestmark = pytest.mark.gpu
S_H = float(np.float32(1) / np.float32(7))
S_H8 = float(np.float32(1) / np.float32(127))


def _tiled8_blob(codes, gates):
    """The 8-bit TILED / TILED_GATES blob written out from the layout notes of the header, in numpy."""
    rows, cols = codes.shape
    H = rows // 4
    rp = (rows + 63) // 64 * 64 if gates else (rows + 15) // 16 * 16
    nkc = (cols + 127) // 128
    padded = np.zeros((rp, nkc * 128), np.int8)
    if gates:
        for j in range(H):
            q, a, b = j // 16, (j % 16) // 4, j % 4
            for g in range(4):
                padded[64 * q + 16 * b + 4 * a + g, :cols] = codes[g * H + j]
    else:
        padded[:rows, :cols] = codes
    blob = np.zeros((rp // 16, nkc, 2, 64, 16), np.int8)
    for lane in range(64):
        r, kq = lane % 16, lane // 16
        rowsel = padded[r::16, :].reshape(rp // 16, nkc, 128)
        for half in range(2):
            blob[:, :, half, lane, :] = rowsel[:, :, 64 * half + 16 * kq:64 * half + 16 * kq + 16]
    return blob.reshape(-1).view(np.uint8)


@pytest.mark.parametrize("rows,cols", [(64, 32), (2560, 352), (46, 256), (4, 16), (256, 1280)])
def test_pack_int8_layout_roundtrip_and_quantizer(gpu_lib, rows, cols):
    q = gpu_lib
    codes = synth.codes(15 + rows + cols, (rows, cols), -128, 127)
    for layout in (q.LAYOUT_ROWMAJOR, q.LAYOUT_TILED) + ((q.LAYOUT_TILED_GATES,) if rows % 4 == 0 else ()):
        m = q.pack_int8(dev(codes), layout)
        assert m.packed.numel() == q.pack_bytes(rows, cols, layout, 8) == 2 * q.pack_bytes(rows, cols, layout, 4)
        assert np.array_equal(host(q.unpack_int4(m)), codes), f"layout {layout}"
        if layout == q.LAYOUT_ROWMAJOR:
            cp = (cols + 63) // 64 * 64
            ref = np.zeros((rows, cp), np.int8); ref[:, :cols] = codes
            assert np.array_equal(host(m.packed).view(np.int8).reshape(rows, cp), ref)
        else:
            assert np.array_equal(host(m.packed), _tiled8_blob(codes, layout == q.LAYOUT_TILED_GATES))
    w = synth.normal(21 + rows, (rows, cols), 1.0 / np.sqrt(cols))
    w[1 % rows, :] = 0.0
    ref_codes, ref_scale = oracle.quantize_weight_rows(w, 8)
    m = q.pack_int8(dev(w), q.LAYOUT_TILED)
    assert np.array_equal(host(q.unpack_int4(m)), ref_codes) and np.array_equal(host(m.row_scale), ref_scale)
    assert np.abs(ref_codes.astype(int)).max() == 127


def test_quantize_act8_bit_exact_including_ties(gpu_lib):
    q = gpu_lib
    x = synth.normal(31, (64 * 3 * 352 + 3,), 1.5)
    inv = float(np.float32(127) / np.float32(4))
    x[:9] = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 1000.0, -1000.0, 0.0, 126.5], np.float32) / np.float32(inv)
    n = x.size - 3
    for sl in (slice(0, 5), slice(0, n - 1), slice(0, n)):
        got = host(q.quantize_act8(dev(x[sl]), inv))
        assert np.array_equal(got, oracle.quant_sym(x[sl], inv, 8))
    assert got.min() == -128 and got.max() == 127


@pytest.mark.parametrize("rows,cols,N,lsm,a8", [(256, 1280, 300, False, False), (256, 768, 16, False, False),
                                                (46, 256, 37, True, True), (32, 64, 5, False, True), (30, 96, 33, False, True)])
def test_linear_int8_weights_parity(gpu_lib, rows, cols, N, lsm, a8):
    """8-bit weights against 4-bit input codes (a cell's output codes) and against 8-bit input codes."""
    q = gpu_lib
    w = synth.normal(41 + rows, (rows, cols), 1.0 / np.sqrt(cols))
    b = synth.normal(42 + rows, (rows,), 0.1)
    a = synth.codes(43 + N, (N, cols), -128, 127) if a8 else synth.codes(43 + N, (N, cols), -8, 7)
    s_a = S_H8 if a8 else S_H
    P = oracle.Linear.from_float(w, b, s_a, bits=8)
    m = q.pack_int8(dev(w), q.LAYOUT_TILED)
    y, acc = q.linear(m, dev(b), s_a, dev(a), log_softmax=lsm, want_acc=True)
    ry, racc = oracle.linear(P, a, want_acc=True)
    assert np.array_equal(host(acc), racc)
    if lsm:
        assert np.abs(host(y) - oracle.log_softmax(ry)).max() < 2e-5
    else:
        assert_rel(host(y), ry, "linear y")
    if not lsm:
        inv = float(np.float32(127.0) / np.float32(0.8))
        got = host(q.linear_quant(m, dev(b), s_a, dev(a), inv, bits=8))
        assert_codes_close(got, oracle.quant_sym(ry, inv, 8), ry.astype(np.float64) * inv, "8-bit codes of y", 0.999)
        assert np.abs(got.astype(int)).max() > 7


@pytest.mark.parametrize("N,J,V,TB", [(4, 32, 16, 40), (1024, 256, 46, 32000), (37, 256, 46, 100)])
def test_joint_fuse_int8_output_layer_parity(gpu_lib, N, J, V, TB):
    """Joint with an 8-bit output layer: z is quantized with 127 steps per side (Sec. 3.2)."""
    q = gpu_lib
    e = synth.normal(81 + N, (TB, J), 1.0)
    p = synth.normal(82 + N, (N, J), 1.0)
    fr = np.random.default_rng(83 + N).integers(0, TB, N).astype(np.int32)
    w = synth.normal(84 + N, (V, J), 1.0 / np.sqrt(J) * 3)
    b = synth.normal(85 + N, (V,), 0.1)
    ls, le = synth.log_probs(86 + N, N, V), synth.log_probs(87 + N, N, V)
    out = oracle.Linear.from_float(w, b, S_H8, bits=8)
    m = q.pack_int8(dev(w), q.LAYOUT_TILED)
    fused, lp, zq = q.joint_fuse(dev(e), dev(fr), dev(p), m, dev(b), dev(ls), dev(le), 0.5, 0.7, rho=0.2,
                                 z_scale=S_H8, z_inv_scale=127.0, want_lp=True, want_zq=True)
    zq_r, z_real = oracle.joint_z(e, fr, p, 127.0, bits=8)
    assert_codes_close(host(zq), zq_r, z_real * 127.0, "z codes", 0.999)
    assert np.abs(host(zq).astype(int)).max() > 100
    lp_r, f_r = oracle.joint_out(out, host(zq), ls, le, 0.5, 0.7, rho=0.2, blank=0)
    assert np.abs(host(lp) - lp_r).max() < 2e-5 and np.abs(host(fused) - f_r).max() < 2e-5


def _lstm8_pair(q, seed, I, H, s_x):
    w_ih = synth.normal(seed, (4 * H, I), 1.0 / np.sqrt(I))
    w_hh = synth.normal(seed + 1, (4 * H, H), 1.0 / np.sqrt(H))
    bias = synth.normal(seed + 2, (4 * H,), 0.1)
    L = oracle.Lstm.from_float(w_ih, w_hh, bias, s_x, S_H8, 127.0, bits=8)
    G = q.Lstm(q.pack_int8(dev(w_ih), q.LAYOUT_TILED_GATES), q.pack_int8(dev(w_hh), q.LAYOUT_TILED_GATES), dev(bias),
               s_x, S_H8, 127.0)
    return L, G


@pytest.mark.parametrize("I,H,M", [(352, 640, 77), (240, 640, 300), (64, 16, 5), (1280, 640, 130)])
def test_input_projection_int8_exact(gpu_lib, I, H, M):
    q = gpu_lib
    L, G = _lstm8_pair(q, 171 + I, I, H, 0.03)
    x = synth.codes(172 + M, (M, I), -128, 127)
    gx, acc = q.input_projection(G, dev(x), debug=True)
    ref = oracle.matmul_i32(L.w_ih, x)
    assert np.array_equal(host(acc), ref)
    col = _tiled_gate_col(H)
    gxh = host(gx)
    for g in range(4):
        assert np.array_equal(gxh[:, col[g]], ref[:, g * H:(g + 1) * H]), f"gate {g}"


@pytest.mark.parametrize("T,B,I,H,reverse", [(20, 2, 32, 64, False), (7, 3, 32, 64, True), (12, 32, 352, 640, False),
                                             (9, 17, 352, 640, True), (5, 120, 64, 640, False)])
def test_lstm_layer_int8_parity(gpu_lib, T, B, I, H, reverse):
    """The 8-bit layer (8-bit weights, inputs and hidden state): GEMM bit-exact, then every step against one
    oracle step fed the GPU's own previous state."""
    q = gpu_lib
    s_x = float(np.float32(4) / np.float32(127))
    L, G = _lstm8_pair(q, 271 + I + H, I, H, s_x)
    x = synth.codes(272 + T, (T, B, I), -128, 127)
    need = q.lstm_layer_workspace(G, T, B)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = q.lstm_layer(G, dev(x), reverse=reverse, want_last=True, debug=True, workspace=ws)
    assert q.layer_error_flag(ws, need) == 0
    hg = host(out["h_out"]); cg = host(out["c_all"])
    assert np.array_equal(host(out["accx"]).reshape(T * B, 4 * H), oracle.matmul_i32(L.w_ih, x.reshape(T * B, I)))
    order = range(T - 1, -1, -1) if reverse else range(T)
    hp = np.zeros((B, H), np.int8); cp = np.zeros((B, H), np.float32)
    for t in order:
        hr, cr, dbg = oracle.lstm_step(L, x[t], hp, cp, debug=True)
        assert_rel(cg[t], cr, f"c t={t}")
        assert_codes_close(hg[t], hr, dbg["h_real"] * 127.0, f"h t={t}", 0.999)
        hp, cp = hg[t], cg[t]
    assert np.abs(hg.astype(int)).max() > 7
    assert np.array_equal(host(out["h_last"]), hp) and np.array_equal(host(out["c_last"]), cp)


def test_step_entry_points_refuse_8bit_layers(gpu_lib):
    q = gpu_lib
    _, G = _lstm8_pair(q, 371, 64, 64, 0.03)
    N = 4
    with pytest.raises(q.QrnntError):
        q.lstm_step(G, dev(synth.codes(1, (N, 64))), dev(synth.codes(2, (N, 64))), dev(synth.normal(3, (N, 64), 0.5)))


@pytest.mark.parametrize("cfg,T,B,W,max_sym", [(0, 12, 2, 4, 2), (5, 3, 2, 4, 2)])
def test_mixed_precision_end_to_end(gpu_lib, cfg, T, B, W, max_sym):
    """The precision map of Sec. 3.2 end to end (8-bit features, first encoder layer, encoder projection,
    prediction-network output layer and joint output layer; everything else 4-bit) against the oracle:
    encoder codes, projection and decoded beams."""
    from paper_2206_07882_amd import model as gmodel
    m = synth.make_model(cfg, mixed=True, weight_std=0.5) if cfg == 0 else synth.make_model(cfg, mixed=True, enc_layers=2)
    feats = synth.features(cfg, T, B, m.feat_dim)
    layers, proj = omodels.encoder_from_float(m)
    x_r, e_r = omodels.encoder_forward(layers, proj, feats, m.alpha_x)
    enc = gmodel.Encoder(m, DEV)
    x_g, e_g = enc.forward(dev(feats))
    agree = (host(x_g) == x_r).mean()
    assert agree >= 0.999, agree
    if agree == 1.0:
        assert np.abs(host(e_g) - e_r).max() < 1e-5
    # decode from the oracle's projection so that an encoder tie cannot leak into the search comparison
    ref = oracle.decode(omodels.model_from_float(m), e_r, W, max_sym)
    got = gpu_lib.decode(gmodel.model_from_float(m, DEV), dev(e_r), W, max_sym)
    _compare_beams(got, ref)
