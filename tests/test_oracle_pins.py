"""Pins of the CPU oracle against things other than itself.

Each test fixes one part of ``oracle/`` with a closed form, an invariant, a
hand-computed value, brute force in plain Python, or a special case that
reduces to a numpy routine, chosen so that a plausible slip (dropped term,
wrong sign, swapped gate, transposed operand) fails at least one of them.
Citations: Sec. 3.1 (quantizers, Eq. 2-3), Sec. 3.2 (what is quantized),
Sec. 3.4 (Outer quantization and its call counts), Sec. 2 (network, Eq. 1).
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from oracle import models

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Sec. 3.1

def test_sym4_clip_range_and_grid_identity():
    # codes never leave [-8, 7]; every grid value is a fixed point of Q o deq
    x = np.linspace(-10, 10, 4001, dtype=np.float32)
    q = oracle.quant_sym4(x, 7.0)
    assert q.min() == -8 and q.max() == 7
    for alpha in (1.0, 1.25, 4.0, 0.37):
        s = np.float32(alpha) / np.float32(7)
        inv = np.float32(7) / np.float32(alpha)
        codes = np.arange(-8, 8, dtype=np.int8)
        back = oracle.quant_sym4(codes.astype(np.float32) * s, inv)
        assert np.array_equal(back, codes)


def test_sym4_zero_maps_to_zero_exactly():
    # symmetric LQ maps a zero input exactly to integer zero (Sec. 3.1)
    assert oracle.quant_sym4(np.array([0.0, -0.0], np.float32), 7.0).tolist() == [0, 0]


def test_sym4_round_half_even_hand_values():
    # x*7 = .5, 1.5, 2.5, -0.5, -1.5, 6.5, 7.5(clipped), -7.5, -8.5(clipped)
    t = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 6.5, 7.5, -7.5, -8.5, 3.49, 3.51], np.float32)
    q = oracle.quant_sym4(t, 1.0)
    assert q.tolist() == [0, 2, 2, 0, -2, 6, 7, -8, -8, 3, 4]


def test_sym4_residual_bound_and_monotone():
    # inside the clipping range the residual is at most s/2 (Sec. 3.1)
    rng = np.random.default_rng(1)
    alpha = 1.25
    s = np.float32(alpha) / np.float32(7)
    inv = np.float32(7) / np.float32(alpha)
    x = rng.uniform(-alpha, alpha, 20000).astype(np.float32)
    q = oracle.quant_sym4(x, inv)
    assert np.all(np.abs(x.astype(np.float64) - q * float(s)) <= float(s) / 2 * (1 + 1e-5))
    xs = np.sort(x)
    assert np.all(np.diff(oracle.quant_sym4(xs, inv).astype(int)) >= 0)


def test_asym_eq2_eq3_worked_example():
    # b=4, alpha=+-1: s = 2/15, z = 7.5 (the worked numbers that follow from Eq. 2-3)
    xi, xq = oracle.quantize_asym(np.array([-1.0, 1.0, 0.0, 5.0, -5.0], np.float32), 4, -1.0, 1.0)
    assert xi[0] == 0 and xi[1] == 15        # alpha_- -> 0, alpha_+ -> 2^b - 1
    assert xi[3] == 15 and xi[4] == 0        # clamp
    assert abs(xq[0] + 1.0) < 1e-12 and abs(xq[1] - 1.0) < 1e-12
    # b=8, asymmetric range with an integer zero point: s=0.01, z=100
    xi, xq = oracle.quantize_asym(np.array([-1.0, 0.0, 0.5, 1.55], np.float32), 8, -1.0, 1.55)
    assert xi.tolist() == [0, 100, 150, 255]
    rng = np.random.default_rng(2)
    x = rng.uniform(-1.0, 1.55, 5000).astype(np.float32)
    _, xq = oracle.quantize_asym(x, 8, -1.0, 1.55)
    assert np.all(np.abs(xq - x) <= 0.005 * (1 + 1e-6))


def test_weight_rows_max_abs_scale_hand_row():
    w = np.array([[0.7, -0.35, 0.05, 0.0, -0.7, 0.1499],
                  [0.0, 0.0, 0.0, 0.0, 0.0, 0.0],
                  [-3.5, 1.0, 0.25, 0.26, 3.0, 0.75]], np.float32)
    q, s = oracle.quantize_weight_rows(w)
    # row 0: alpha=.7, step .1 -> 7, -3.5->-4 (tie to even), .5->0 (tie to even), 0, -7, 1.499->1
    assert q[0].tolist() == [7, -4, 0, 0, -7, 1]
    assert abs(s[0] - 0.1) < 1e-7
    assert q[1].tolist() == [0] * 6 and s[1] == 1.0
    # row 2: alpha=3.5, step .5 -> -7, 2, .5->0, .52->1, 6, 1.5->2
    assert q[2].tolist() == [-7, 2, 0, 1, 6, 2]
    rng = np.random.default_rng(3)
    w = rng.standard_normal((50, 33)).astype(np.float32)
    q, s = oracle.quantize_weight_rows(w)
    assert np.all(np.abs(q).max(axis=1) == 7) and q.min() >= -7
    assert np.allclose(s, np.abs(w).max(axis=1) / 7, rtol=1e-6)


def test_pack_hand_bytes_and_roundtrip_all_bytes():
    codes = np.array([[1, -1, 7, -8, 0, 3]], np.int8)
    p = oracle.pack_rows(codes, 8)
    assert p.tolist() == [[0xF1, 0x87, 0x30, 0x00]]
    # all 256 byte values: every (lo, hi) nibble pair
    lo, hi = np.meshgrid(np.arange(-8, 8), np.arange(-8, 8))
    allc = np.stack([lo.ravel(), hi.ravel()], axis=1).astype(np.int8).reshape(1, -1)
    p = oracle.pack_rows(allc, allc.shape[1])
    assert sorted(p.ravel().tolist()) == list(range(256))
    assert np.array_equal(oracle.unpack_rows(p, allc.shape[1]), allc)
    # ragged: cols 5 padded to 8
    c5 = np.array([[1, 2, 3, 4, 5], [-1, -2, -3, -4, -5]], np.int8)
    p = oracle.pack_rows(c5, 8)
    assert p.shape == (2, 4) and p[0].tolist() == [0x21, 0x43, 0x05, 0x00]
    assert np.array_equal(oracle.unpack_rows(p, 5), c5)


# ------------------------------------------------------------------ integer MAC

def test_matmul_bruteforce_and_extremes():
    rng = np.random.default_rng(4)
    w = rng.integers(-8, 8, (5, 7)).astype(np.int8)
    a = rng.integers(-8, 8, (3, 7)).astype(np.int8)
    ref = [[sum(int(w[r, k]) * int(a[n, k]) for k in range(7)) for r in range(5)] for n in range(3)]
    assert oracle.matmul_i32(w, a).tolist() == ref
    K = 2048
    assert oracle.matmul_i32(np.full((2, K), -8, np.int8), np.full((1, K), -8, np.int8)).tolist() == [[64 * K] * 2]
    assert oracle.matmul_i32(np.full((2, K), 7, np.int8), np.full((1, K), -8, np.int8)).tolist() == [[-56 * K] * 2]
    w = rng.integers(-8, 8, (9, 300)).astype(np.int8)
    a = rng.integers(-8, 8, (4, 300)).astype(np.int8)
    perm = rng.permutation(300)
    assert np.array_equal(oracle.matmul_i32(w, a), oracle.matmul_i32(w[:, perm], a[:, perm]))
    assert np.array_equal(oracle.matmul_i32(w, a), a.astype(np.int64) @ w.astype(np.int64).T)


# ------------------------------------------------------------------ LSTM cell

def _rand_lstm(rng, I, H, s_x=0.2):
    return oracle.Lstm(rng.integers(-7, 8, (4 * H, I)), rng.uniform(0.005, 0.03, 4 * H),
                       rng.integers(-7, 8, (4 * H, H)), rng.uniform(0.005, 0.03, 4 * H),
                       rng.standard_normal(4 * H) * 0.3, s_x)


def test_lstm_zero_weights_closed_form():
    # zero weights: i,f,o = sigma(b), g = tanh(b); c_t = i g (1 - f^t)/(1 - f); h_t = o tanh(c_t)
    H, I, T, B = 6, 5, 25, 2
    rng = np.random.default_rng(5)
    b = rng.standard_normal(4 * H)
    L = oracle.Lstm(np.zeros((4 * H, I)), np.ones(4 * H), np.zeros((4 * H, H)), np.ones(4 * H), b, 0.3)
    x = rng.integers(-7, 8, (T, B, I)).astype(np.int8)
    h_out, h_last, c_last, c_all = oracle.lstm_layer(L, x, want_c_all=True)
    b32 = b.astype(np.float32).astype(np.float64)
    sg = lambda v: 1 / (1 + np.exp(-v))
    i, f, g, o = sg(b32[:H]), sg(b32[H:2 * H]), np.tanh(b32[2 * H:3 * H]), sg(b32[3 * H:])
    for t in range(1, T + 1):
        c = i * g * (1 - f ** t) / (1 - f)
        assert np.allclose(c_all[t - 1, 0], c, rtol=2e-6, atol=1e-7)   # fp32 storage of c each step
        h = o * np.tanh(c)
        code = np.rint(h * 7)
        near_tie = np.abs(h * 7 - np.floor(h * 7) - 0.5) < 1e-4
        assert np.all((h_out[t - 1, 1] == code) | near_tie)


def test_lstm_step_against_numpy_cell():
    # an independent restatement with numpy: dequantize, float matmul, textbook LSTM
    rng = np.random.default_rng(6)
    I, H, N = 24, 16, 9
    L = _rand_lstm(rng, I, H)
    x = rng.integers(-8, 8, (N, I)).astype(np.int8)
    hp = rng.integers(-7, 8, (N, H)).astype(np.int8)
    cp = rng.standard_normal((N, H)).astype(np.float32)
    hn, cn, dbg = oracle.lstm_step(L, x, hp, cp, debug=True)
    Wih = L.w_ih.astype(np.float64) * L.s_wih.astype(np.float64)[:, None]
    Whh = L.w_hh.astype(np.float64) * L.s_whh.astype(np.float64)[:, None]
    pre = (x.astype(np.float64) * float(L.s_x)) @ Wih.T + (hp.astype(np.float64) * float(L.s_h)) @ Whh.T + L.bias
    sg = lambda v: 1 / (1 + np.exp(-v))
    gi, gf, gg, go = sg(pre[:, :H]), sg(pre[:, H:2 * H]), np.tanh(pre[:, 2 * H:3 * H]), sg(pre[:, 3 * H:])
    c = gf * cp + gi * gg
    h = go * np.tanh(c)
    assert np.allclose(dbg["gates"], np.concatenate([gi, gf, gg, go], 1), rtol=1e-12, atol=1e-13)
    assert np.allclose(cn, c, rtol=1e-6, atol=1e-7)
    assert np.allclose(dbg["h_real"], h, rtol=1e-9, atol=1e-12)
    tie = np.abs(h * 7 - np.floor(h * 7) - 0.5) < 1e-5
    assert np.all((hn == np.rint(h * 7)) | tie)
    assert np.array_equal(dbg["accx"], x.astype(np.int64) @ L.w_ih.astype(np.int64).T)
    assert np.array_equal(dbg["acch"], hp.astype(np.int64) @ L.w_hh.astype(np.int64).T)
    assert np.abs(hn).max() <= 7    # h = tanh * sigma is in [-1,1]: FIX +-1 never clips (Sec. 3.2)


def test_8bit_quantizers_range_grid_and_hand_values():
    # Sec. 3.2 keeps the first encoder layer and the RNN-T's linear layers at 8 bits (MAX for weights
    # and inputs, FIX +-1 for hidden states): the same symmetric quantizer with 2^7 - 1 = 127 steps per side.
    rng = np.random.default_rng(61)
    x = (rng.standard_normal(4000) * 2).astype(np.float32)
    for inv in (7.0, 3.3):
        assert np.array_equal(oracle.quant_sym(x, inv, 4), oracle.quant_sym4(x, inv))      # b = 4 is the 4-bit routine
    inv = np.float32(127.0)                                                                 # FIX +-1 at 8 bits
    q = oracle.quant_sym(x, inv, 8)
    assert q.min() == -128 and q.max() == 127                                               # clip range
    codes = np.arange(-128, 128, dtype=np.float32)
    assert np.array_equal(oracle.quant_sym(codes * (np.float32(1) / inv), inv, 8), codes.astype(np.int8))  # grid identity
    assert oracle.quant_sym(np.zeros(1, np.float32), inv, 8)[0] == 0
    hand = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 126.5, 127.5, 300.0, -128.5, -129.5], np.float32) / inv
    assert oracle.quant_sym(hand, inv, 8).tolist() == [0, 2, 2, 0, -2, 126, 127, 127, -128, -128]     # ties to even, clamp
    inside = np.abs(x) < 0.99
    assert np.abs(q[inside] / 127.0 - x[inside]).max() <= 0.5 / 127 + 1e-6                  # residual <= s/2
    # weights: per-row MAX at 8 bits
    w = (rng.standard_normal((5, 33)) * np.array([0.01, 0.3, 1.0, 5.0, 0.0])[:, None]).astype(np.float32)
    c8, s8 = oracle.quantize_weight_rows(w, 8)
    c4, s4 = oracle.quantize_weight_rows(w, 4)
    assert np.array_equal(np.abs(c8[:4]).max(1), [127] * 4) and np.array_equal(np.abs(c4[:4]).max(1), [7] * 4)
    assert np.array_equal(c8[4], np.zeros(33)) and s8[4] == 1.0
    assert np.allclose(s8[:4], np.abs(w[:4]).max(1) / 127, rtol=1e-6)
    assert np.all(np.abs(c8[:4] * s8[:4, None] - w[:4]) <= s8[:4, None] * 0.5 * (1 + 1e-5))
    assert np.abs(c8[:4] * s8[:4, None] - w[:4]).max() < np.abs(c4[:4] * s4[:4, None] - w[:4]).max() / 8
    row = np.array([[0.5, -1.0, 0.25, 1.0 / 127 * 1.5, 0.0]], np.float32)
    assert oracle.quantize_weight_rows(row, 8)[0].tolist() == [[64, -127, 32, 2, 0]]      # 63.5 -> 64, 31.75 -> 32, 1.5 -> 2


def test_8bit_lstm_layer_and_joint_against_numpy():
    # the hidden-state quantizer of an 8-bit layer has 127 steps per side; everything else is the same cell
    rng = np.random.default_rng(62)
    I, H, N = 24, 16, 9
    L = oracle.Lstm.from_float((rng.standard_normal((4 * H, I)) * 0.3).astype(np.float32),
                               (rng.standard_normal((4 * H, H)) * 0.3).astype(np.float32),
                               (rng.standard_normal(4 * H) * 0.1).astype(np.float32),
                               np.float32(4.0 / 127), np.float32(1.0) / np.float32(127.0), 127.0, bits=8)
    assert np.abs(L.w_ih).max() == 127
    x = rng.integers(-128, 128, (N, I)).astype(np.int8)
    hp = rng.integers(-127, 128, (N, H)).astype(np.int8)
    cp = rng.standard_normal((N, H)).astype(np.float32)
    hn, cn, dbg = oracle.lstm_step(L, x, hp, cp, debug=True)
    Wih = L.w_ih.astype(np.float64) * L.s_wih.astype(np.float64)[:, None]
    Whh = L.w_hh.astype(np.float64) * L.s_whh.astype(np.float64)[:, None]
    pre = (x.astype(np.float64) * float(L.s_x)) @ Wih.T + (hp.astype(np.float64) * float(L.s_h)) @ Whh.T + L.bias
    sg = lambda v: 1 / (1 + np.exp(-v))
    gi, gf, gg, go = sg(pre[:, :H]), sg(pre[:, H:2 * H]), np.tanh(pre[:, 2 * H:3 * H]), sg(pre[:, 3 * H:])
    c = gf * cp + gi * gg
    h = go * np.tanh(c)
    assert np.allclose(cn, c, rtol=1e-6, atol=1e-7)
    tie = np.abs(h * 127 - np.floor(h * 127) - 0.5) < 1e-4
    assert np.all((hn == np.rint(h * 127)) | tie) and np.abs(hn.astype(int)).max() > 7
    assert np.array_equal(dbg["accx"], x.astype(np.int64) @ L.w_ih.astype(np.int64).T)
    # joint with an 8-bit output layer: z is quantized with 127 steps per side
    e, p, fr, out4, ls, le = _joint_setup(rng)
    out8 = oracle.Linear.from_float(out4.w * out4.s_w[:, None], out4.bias, np.float32(1.0) / np.float32(127.0), bits=8)
    zq, lp, _ = oracle.joint_fuse(e, fr, p, out8, None, None, 0.0, 0.0, inv_s_z=127.0)
    z = np.tanh(e[fr].astype(np.float64) * p.astype(np.float64))
    tie = np.abs(z * 127 - np.floor(z * 127) - 0.5) < 1e-4
    assert np.all((zq == np.rint(z * 127)) | tie) and np.abs(zq.astype(int)).max() > 7
    logits = (zq.astype(np.float64) * float(out8.s_a)) @ (out8.w * out8.s_w.astype(np.float64)[:, None]).T + out8.bias
    assert np.allclose(lp, logits - np.log(np.exp(logits).sum(1, keepdims=True)), atol=1e-5)


def test_lstm_gate_roles_by_saturation():
    # saturating one gate at a time shows each block of rows plays its textbook role
    H, I = 4, 3
    big = 40.0
    x = np.zeros((1, I), np.int8); hp = np.zeros((1, H), np.int8)
    cp = np.full((1, H), 0.5, np.float32)

    def run(bi, bf, bg, bo):
        b = np.concatenate([np.full(H, bi), np.full(H, bf), np.full(H, bg), np.full(H, bo)])
        L = oracle.Lstm(np.zeros((4 * H, I)), np.ones(4 * H), np.zeros((4 * H, H)), np.ones(4 * H), b, 1.0)
        return oracle.lstm_step(L, x, hp, cp)

    hn, cn = run(-big, big, big, big)      # input gate closed, forget open: c stays
    assert np.allclose(cn, 0.5)
    hn, cn = run(big, -big, big, big)      # forget closed, input open, g=+1: c = 1
    assert np.allclose(cn, 1.0)
    hn, cn = run(big, -big, -big, big)     # g = -1
    assert np.allclose(cn, -1.0)
    assert hn.tolist() == [[int(np.rint(math.tanh(-1.0) * 7))] * H]
    hn, cn = run(big, -big, big, -big)     # output gate closed: h = 0
    assert hn.tolist() == [[0] * H]


def test_lstm_parent_gather_and_inactive_passthrough():
    rng = np.random.default_rng(7)
    I, H, N = 8, 8, 6
    L = _rand_lstm(rng, I, H)
    x = rng.integers(-7, 8, (N, I)).astype(np.int8)
    hp = rng.integers(-7, 8, (N, H)).astype(np.int8)
    cp = rng.standard_normal((N, H)).astype(np.float32)
    parent = np.array([3, 3, 0, 5, 1, 1], np.int32)
    active = np.array([1, 0, 1, 1, 0, 1], np.uint8)
    hn, cn = oracle.lstm_step(L, x, hp, cp, parent=parent, active=active)
    hn2, cn2 = oracle.lstm_step(L, x, hp[parent], cp[parent])
    for n in range(N):
        if active[n]:
            assert np.array_equal(hn[n], hn2[n]) and np.array_equal(cn[n], cn2[n])
        else:
            assert np.array_equal(hn[n], hp[parent[n]]) and np.array_equal(cn[n], cp[parent[n]])


def test_lstm_layer_reverse_is_time_flip_and_offsets():
    rng = np.random.default_rng(8)
    I, H, T, B = 10, 8, 7, 3
    L = _rand_lstm(rng, I, H)
    x = rng.integers(-7, 8, (T, B, I)).astype(np.int8)
    fwd_on_flipped, _, _, _ = oracle.lstm_layer(L, x[::-1].copy())
    out = np.full((T, B, 2 * H + 3), 99, np.int8)
    oracle.lstm_layer(L, x, reverse=True, h_out=out, col_off=H)
    assert np.array_equal(out[:, :, H:2 * H], fwd_on_flipped[::-1])
    assert np.all(out[:, :, :H] == 99) and np.all(out[:, :, 2 * H:] == 99)
    # T = 1 equals one step from the zero state
    h1, hl, cl, _ = oracle.lstm_layer(L, x[:1])
    hs, cs = oracle.lstm_step(L, x[0], np.zeros((B, H), np.int8), np.zeros((B, H), np.float32))
    assert np.array_equal(h1[0], hs) and np.array_equal(cl, cs) and np.array_equal(hl, hs)


def test_outer_quantization_call_counts():
    # Sec. 3.4: Outer needs T + T*L quantizer calls, Inner 2*T*L; ratio (L+1)/(2L);
    # L = 12 (6 bidirectional layers counted twice) gives 13/24, i.e. about 45 % fewer calls.
    rng = np.random.default_rng(9)
    T, B, D, H, layers = 5, 2, 6, 4, 3
    L_dirs = 2 * layers
    feats = rng.standard_normal((T, B, D)).astype(np.float32)
    oracle.quant_calls_reset()
    x = np.stack([oracle.quant_sym4(feats[t], 7 / 4) for t in range(T)])    # one call per time step
    for l in range(layers):
        I = D if l == 0 else 2 * H
        out = np.zeros((T, B, 2 * H), np.int8)
        for d in range(2):
            oracle.lstm_layer(_rand_lstm(rng, I, H), x, reverse=bool(d), h_out=out, col_off=d * H)
        x = out        # the stored codes feed the next layer: no second quantizer
    assert oracle.quant_calls() == T + T * L_dirs
    assert (T + T * L_dirs) / (2 * T * L_dirs) == (L_dirs + 1) / (2 * L_dirs)
    assert abs((1 - 13 / 24) - 0.458) < 1e-3


# ------------------------------------------------------------------ linear, joint, Eq. 1

def test_linear_against_dequantized_float_matmul():
    rng = np.random.default_rng(10)
    w = rng.integers(-8, 8, (11, 40)).astype(np.int8)
    sw = rng.uniform(0.01, 0.05, 11).astype(np.float32)
    b = rng.standard_normal(11).astype(np.float32)
    P = oracle.Linear(w, sw, b, 1 / 7)
    a = rng.integers(-8, 8, (6, 40)).astype(np.int8)
    y, acc = oracle.linear(P, a, want_acc=True)
    ref = (a.astype(np.float64) * float(np.float32(1 / 7))) @ (w.astype(np.float64) * sw.astype(np.float64)[:, None]).T + b
    assert np.allclose(y, ref, rtol=1e-6, atol=1e-6)
    assert np.array_equal(acc, a.astype(np.int64) @ w.astype(np.int64).T)


def test_log_softmax_properties():
    rng = np.random.default_rng(11)
    x = (rng.standard_normal((7, 46)) * 5).astype(np.float32)
    lp = oracle.log_softmax(x)
    assert np.allclose(np.exp(lp.astype(np.float64)).sum(1), 1.0, atol=1e-6)
    assert np.allclose(oracle.log_softmax(x + np.float32(100.0)), lp, atol=2e-5)
    assert np.allclose(oracle.log_softmax(np.full((1, 46), 3.0, np.float32)), -math.log(46), atol=1e-6)
    assert np.allclose(lp[:, 1:] - lp[:, :1], (x[:, 1:] - x[:, :1]), atol=1e-5)   # differences preserved
    big = np.array([[1000.0, 0.0, -1000.0]], np.float32)                        # no overflow
    assert np.allclose(oracle.log_softmax(big), [[0.0, -1000.0, -2000.0]])


def _joint_setup(rng, N=5, J=16, V=7, TB=4):
    e = rng.standard_normal((TB, J)).astype(np.float32)
    p = rng.standard_normal((N, J)).astype(np.float32)
    fr = rng.integers(0, TB, N).astype(np.int32)
    out = oracle.Linear(rng.integers(-7, 8, (V, J)), rng.uniform(0.05, 0.2, V), rng.standard_normal(V) * 0.2, 1 / 7)
    ls = np.log(rng.dirichlet(np.ones(V), N)).astype(np.float32)
    le = np.log(rng.dirichlet(np.ones(V), N)).astype(np.float32)
    return e, p, fr, out, ls, le


def test_joint_against_numpy_restatement():
    rng = np.random.default_rng(12)
    e, p, fr, out, ls, le = _joint_setup(rng)
    zq, lp, fused = oracle.joint_fuse(e, fr, p, out, ls, le, 0.3, 0.5, rho=0.2, blank=0)
    z = np.tanh(e[fr].astype(np.float64) * p.astype(np.float64))      # multiplicative combination (Sec. 2)
    tie = np.abs(z * 7 - np.floor(z * 7) - 0.5) < 1e-5
    assert np.all((zq == np.rint(z * 7)) | tie) and np.abs(zq).max() <= 7
    logits = (zq.astype(np.float64) * float(np.float32(1 / 7))) @ (out.w * out.s_w.astype(np.float64)[:, None]).T + out.bias
    ref_lp = logits - np.log(np.exp(logits).sum(1, keepdims=True))
    assert np.allclose(lp, ref_lp, atol=1e-5)
    ref_f = ref_lp.copy()
    ref_f[:, 1:] += -0.3 * ls[:, 1:].astype(np.float64) + 0.5 * le[:, 1:].astype(np.float64) + 0.2
    assert np.allclose(fused, ref_f, atol=1e-5)
    assert np.allclose(fused[:, 0], lp[:, 0])        # blank is not an LM event


def test_fusion_special_cases_of_eq1():
    rng = np.random.default_rng(13)
    e, p, fr, out, ls, le = _joint_setup(rng)
    _, lp, f0 = oracle.joint_fuse(e, fr, p, out, ls, le, 0.0, 0.0, rho=0.0)
    assert np.array_equal(f0, lp)                                     # lambda = mu = rho = 0: plain RNN-T
    _, _, fn = oracle.joint_fuse(e, fr, p, out, None, None, 0.3, 0.5)
    assert np.array_equal(fn, lp)                                     # no LMs
    _, _, f1 = oracle.joint_fuse(e, fr, p, out, ls, le, 0.4, 0.0)
    _, _, f2 = oracle.joint_fuse(e, fr, p, out, ls, le, 0.8, 0.0)
    assert np.allclose(f2 - f1, f1 - f0, atol=2e-6)                   # affine in lambda_src
    assert np.all((f1 - f0)[:, 1:] > 0)                               # source LM enters with a minus sign (lp<0)
    _, _, g1 = oracle.joint_fuse(e, fr, p, out, ls, le, 0.0, 0.7)
    assert np.allclose((g1 - f0)[:, 1:], 0.7 * le[:, 1:], atol=2e-6)  # external LM enters with a plus sign
    _, _, r1 = oracle.joint_fuse(e, fr, p, out, ls, le, 0.0, 0.0, rho=0.2)
    assert np.allclose((r1 - f0)[:, 1:], 0.2, atol=1e-6) and np.array_equal(r1[:, 0], f0[:, 0])


# ------------------------------------------------------------------ beam selection

def _beam_ref(score, fused, blank, force):
    B, W = score.shape
    V = fused.shape[-1]
    par = np.full((B, W), -1, np.int32); tok = np.full((B, W), -1, np.int32)
    ns = np.full((B, W), -np.inf, np.float32)
    for b in range(B):
        val = (score[b][:, None] + fused.reshape(B, W, V)[b]).astype(np.float32).ravel()
        if force:
            mask = np.ones(W * V, bool); mask[blank::V] = False
            val[mask] = -np.inf
        order = np.lexsort((np.arange(W * V), -val.astype(np.float64)))
        r = 0
        for c in order:
            if r == W or not np.isfinite(val[c]):
                break
            par[b, r], tok[b, r], ns[b, r] = c // V, c % V, val[c]
            r += 1
    return par, tok, ns


def test_beam_step_against_lexsort_with_ties_and_dead_slots():
    rng = np.random.default_rng(14)
    B, W, V = 3, 4, 6
    score = rng.standard_normal((B, W)).astype(np.float32)
    score[1, 2:] = -np.inf                    # dead slots
    score[2, 1:] = -np.inf                    # a single live slot: fewer finite candidates than ... V=6 >= W
    fused = rng.standard_normal((B * W, V)).astype(np.float32)
    fused[0, 1] = fused[0, 3] = 9.0           # exact tie inside one parent -> lower token first
    score[0, 1] = score[0, 0]; fused[1, :] = fused[0, :]    # ties across parents -> lower parent first
    for force in (False, True):
        got = oracle.beam_step(score, fused, blank=0, force_blank=force)
        ref = _beam_ref(score, fused, 0, force)
        for g, r in zip(got, ref):
            assert np.array_equal(g, r)
    par, tok, ns = oracle.beam_step(score, fused)
    assert (par[0, 0], tok[0, 0], par[0, 1], tok[0, 1]) == (0, 1, 0, 3)
    assert (par[0, 2], tok[0, 2], par[0, 3], tok[0, 3]) == (1, 1, 1, 3)
    par, tok, ns = oracle.beam_step(score, fused, force_blank=True)
    assert np.all(tok[np.isfinite(ns)] == 0) and np.sum(np.isfinite(ns[1])) == 2 and np.sum(np.isfinite(ns[2])) == 1
    assert np.all(par[~np.isfinite(ns)] == -1)


# ------------------------------------------------------------------ networks and search

def _tiny_model(seed, V=3, E=6, H=6, J=5, with_lms=True, lam=(0.3, 0.5), rho=0.0, std=0.8):
    rng = np.random.default_rng(seed)

    def net(out_rows, ls):
        L = oracle.Lstm.from_float(rng.standard_normal((4 * H, E)) * std, rng.standard_normal((4 * H, H)) * std,
                                   rng.standard_normal(4 * H) * 0.2, np.float32(1.25) / np.float32(7))
        out = oracle.Linear.from_float(rng.standard_normal((out_rows, H)) * std, rng.standard_normal(out_rows) * 0.2,
                                       np.float32(1) / np.float32(7))
        return oracle.Net(rng.standard_normal((V, E)) * 0.5, 1.25, [L], out, ls)

    pred = net(J, False)
    src = net(V, True) if with_lms else None
    ext = net(V, True) if with_lms else None
    jout = oracle.Linear.from_float(rng.standard_normal((V, J)) * 1.5, rng.standard_normal(V) * 0.3,
                                    np.float32(1) / np.float32(7))
    return oracle.Model(pred, src, ext, jout, lam[0], lam[1], rho)


def _state_outputs(model, tokens):
    """Network outputs after feeding [start symbol 0] + tokens from the zero
    state, recomputed from scratch (independent of the search's state copies)."""
    seq = np.array([0] + list(tokens), np.int32)
    p = oracle.net_run(model.pred, seq)[-1]
    ls = oracle.net_run(model.lm_src, seq)[-1] if model.lm_src is not None else None
    le = oracle.net_run(model.lm_ext, seq)[-1] if model.lm_ext is not None else None
    return p, ls, le


def _fused_row(model, e, T_B_row, tokens):
    p, ls, le = _state_outputs(model, tokens)
    _, _, f = oracle.joint_fuse(e.reshape(-1, e.shape[-1]), np.array([T_B_row], np.int32), p[None], model.joint_out,
                                None if ls is None else ls[None], None if le is None else le[None],
                                model.lambda_src, model.lambda_ext, model.rho, model.blank, model.inv_s_z)
    return f[0]


def test_net_run_matches_manual_steps():
    m = _tiny_model(20)
    net = m.lm_ext
    toks = [0, 2, 1, 1]
    y = oracle.net_run(net, np.array(toks, np.int32))
    h = np.zeros((1, net.layers[0].H), np.int8); c = np.zeros((1, net.layers[0].H), np.float32)
    for i, t in enumerate(toks):
        xq = oracle.quant_sym4(net.embed[t][None], net.inv_s_e)
        h, c = oracle.lstm_step(net.layers[0], xq, h, c)
        ref = oracle.log_softmax(oracle.linear(net.out, h))
        assert np.array_equal(y[i], ref[0])
    assert np.allclose(np.exp(y.astype(np.float64)).sum(1), 1, atol=1e-6)


def test_net_bottleneck_against_float_restatement():
    # Sec. 2 (external LM): LSTM stack -> bottleneck -> output layer -> log-softmax.  The network with a
    # bottleneck must equal, at every step, the same LSTM stack followed by a numpy restatement of the
    # two dequantized matrix products with the quantizer between them.
    rng = np.random.default_rng(33)
    V, E, H, M = 7, 16, 32, 16
    embed = (rng.standard_normal((V, E)) * 0.5).astype(np.float32)
    L = oracle.Lstm.from_float((rng.standard_normal((4 * H, E)) * 0.3).astype(np.float32),
                               (rng.standard_normal((4 * H, H)) * 0.3).astype(np.float32),
                               (rng.standard_normal(4 * H) * 0.1).astype(np.float32), np.float32(1.25 / 7))
    alpha_mid = 0.35
    s_m = np.float32(np.float32(alpha_mid) / np.float32(7))
    mid = oracle.Linear.from_float((rng.standard_normal((M, H)) * 0.4).astype(np.float32),
                                   (rng.standard_normal(M) * 0.1).astype(np.float32), np.float32(1) / np.float32(7))
    out = oracle.Linear.from_float((rng.standard_normal((V, M)) * 0.5).astype(np.float32),
                                   (rng.standard_normal(V) * 0.1).astype(np.float32), s_m)
    net = oracle.Net(embed, 1.25, [L], out, True, mid=mid, alpha_mid=alpha_mid)
    plain = oracle.Net(embed, 1.25, [L], oracle.Linear(np.eye(H, dtype=np.int8), np.ones(H, np.float32), None, 1.0), False)
    toks = np.array([0, 3, 6, 1, 1, 5], np.int32)
    y = oracle.net_run(net, toks)
    h_codes = oracle.net_run(plain, toks)          # identity output layer with unit scales: the top hidden codes
    assert np.array_equal(h_codes, np.rint(h_codes)) and np.abs(h_codes).max() <= 7
    saw_clip = False
    for i in range(len(toks)):
        ym = (mid.w.astype(np.float64) * mid.s_w[:, None].astype(np.float64)) @ (h_codes[i].astype(np.float64) / 7) + mid.bias
        t = ym * float(np.float32(7) / np.float32(alpha_mid))
        if np.abs(np.abs(t - np.floor(t)) - 0.5).min() < 1e-4:
            continue                                # too close to a rounding tie for a float restatement
        qm = np.clip(np.rint(t), -8, 7)
        saw_clip = saw_clip or np.abs(t).max() > 7.5
        yo = (out.w.astype(np.float64) * out.s_w[:, None].astype(np.float64)) @ (qm * float(s_m)) + out.bias
        ref = yo - (np.log(np.exp(yo - yo.max()).sum()) + yo.max())
        assert np.abs(y[i] - ref).max() < 2e-5, i
    assert saw_clip                                 # the quantizer between the layers does clip here
    # without the bottleneck the same network gives other values (the layer is really applied)
    direct = oracle.Net(embed, 1.25, [L], oracle.Linear.from_float(
        (rng.standard_normal((V, H)) * 0.5).astype(np.float32), None, np.float32(1) / np.float32(7)), True)
    assert np.abs(oracle.net_run(direct, toks) - y).max() > 1e-2


def test_beam1_equals_independent_greedy():
    # W = 1 is greedy decoding with a cap on labels per frame
    for seed, lms in ((21, True), (22, False)):
        m = _tiny_model(seed, V=5, with_lms=lms)
        rng = np.random.default_rng(seed)
        T, B, max_sym = 6, 2, 3
        e = rng.standard_normal((T, B, m.joint_out.cols)).astype(np.float32)
        tok, ln, sc = oracle.decode(m, e, 1, max_sym)
        for b in range(B):
            seq, S = [], np.float32(0)
            for t in range(T):
                for v in range(max_sym + 1):
                    f = _fused_row(m, e, t * B + b, seq)
                    k = 0 if v == max_sym else int(np.argmax(f))
                    S = np.float32(S + f[k])
                    if k == 0:
                        break
                    seq.append(k)
            assert ln[b, 0] == len(seq) and tok[b, 0, :len(seq)].tolist() == seq
            assert abs(sc[b, 0] - S) < 1e-4
        assert any(ln[:, 0] > 0)


def test_beam_search_equals_exhaustive_enumeration_when_nothing_is_pruned():
    # T=2 frames, V=3, at most 2 labels per frame: 7 label strings per frame, 49 alignments.
    # With W=64 no candidate is ever dropped, so the search must return every alignment's
    # score, best first; an independent Python enumeration provides them.
    m = _tiny_model(23, V=3)
    rng = np.random.default_rng(23)
    T, B, max_sym, W = 2, 1, 2, 64
    e = rng.standard_normal((T, B, m.joint_out.cols)).astype(np.float32)
    per_frame = [()] + [s for n in (1, 2) for s in itertools.product((1, 2), repeat=n)]
    scores = []
    for f0 in per_frame:
        for f1 in per_frame:
            seq, S = [], np.float32(0)
            for t, labs in enumerate((f0, f1)):
                for k in list(labs) + [0]:
                    S = np.float32(S + _fused_row(m, e, t * B, seq)[k])
                    if k:
                        seq.append(k)
            scores.append((float(S), tuple(seq)))
            acts = list(f0) + [0] + list(f1) + [0]
            assert abs(oracle.score_alignment(m, e, 0, acts) - float(S)) < 1e-5
    scores.sort(key=lambda s: -s[0])
    tok, ln, sc = oracle.decode(m, e, W, max_sym)
    n = int((ln[0] >= 0).sum())
    assert n == len(scores) == 49
    assert np.allclose(sc[0, :n], [s for s, _ in scores], atol=1e-5)
    assert np.all(np.diff(sc[0, :n]) <= 0)
    assert tuple(tok[0, 0, :ln[0, 0]].tolist()) == scores[0][1]
    # a narrow beam can only do worse or equal, never better, than the exhaustive optimum
    tok2, ln2, sc2 = oracle.decode(m, e, 2, max_sym)
    assert sc2[0, 0] <= sc[0, 0] + 1e-6


def test_alsd_without_pruning_sums_over_all_alignments():
    # Alignment-length synchronous search with recombination (the paper's search, Sec. 2): with a beam so wide
    # that nothing is pruned, the final score of a label sequence is the log of its total probability over all
    # alignments (the transducer's forward recursion, restated here in numpy) plus its label-wise terms of Eq. 1.
    import itertools
    for seed, lms in ((41, True), (42, False)):
        m = _tiny_model(seed, V=3, with_lms=lms)
        rng = np.random.default_rng(seed)
        T, B, u_max, W = 3, 2, 2, 200
        e = rng.standard_normal((T, B, m.joint_out.cols)).astype(np.float32)
        tok, ln, sc = oracle.decode_alsd(m, e, W, u_max)
        seqs = [()] + [s for u in (1, 2) for s in itertools.product((1, 2), repeat=u)]
        for b in range(B):
            got = {tuple(tok[b, r, :ln[b, r]]): float(sc[b, r]) for r in range(W) if ln[b, r] >= 0}
            assert sorted(got) == sorted(seqs)                       # every sequence finishes exactly once
            fin = [float(sc[b, r]) for r in range(W) if ln[b, r] >= 0]
            assert fin == sorted(fin, reverse=True)
            for y in seqs:
                U = len(y)
                F = np.stack([np.stack([_fused_row(m, e, t * B + b, list(y[:u])) for u in range(U + 1)])
                              for t in range(T)]).astype(np.float64)   # [t, u, k]
                alpha = np.full((T, U + 1), -np.inf)
                alpha[0, 0] = 0.0
                for t in range(T):
                    for u in range(U + 1):
                        if t > 0:
                            alpha[t, u] = np.logaddexp(alpha[t, u], alpha[t - 1, u] + F[t - 1, u, 0])
                        if u > 0:
                            alpha[t, u] = np.logaddexp(alpha[t, u], alpha[t, u - 1] + F[t, u - 1, y[u - 1]])
                total = alpha[T - 1, U] + F[T - 1, U, 0]
                assert abs(got[y] - total) < 2e-4, (y, got[y], total)
        # u_max = 0: only the all-blank alignment exists
        tok0, ln0, sc0 = oracle.decode_alsd(m, e, 4, 0)
        for b in range(B):
            ref = np.float32(0)
            for t in range(T):
                ref = np.float32(ref + _fused_row(m, e, t * B + b, [])[0])
            assert ln0[b].tolist() == [0, -1, -1, -1] and abs(sc0[b, 0] - ref) < 1e-5


def test_alsd_permuting_utterances_permutes_outputs():
    m = _tiny_model(43, V=5)
    rng = np.random.default_rng(43)
    e = rng.standard_normal((5, 3, m.joint_out.cols)).astype(np.float32)
    a = oracle.decode_alsd(m, e, 4, 6)
    perm = [2, 0, 1]
    p = oracle.decode_alsd(m, np.ascontiguousarray(e[:, perm]), 4, 6)
    for x, y in zip(a, p):
        assert np.array_equal(x[perm], y)
    assert (a[1][:, 0] > 0).any()


def test_decode_permuting_utterances_permutes_outputs():
    m = _tiny_model(24, V=5)
    rng = np.random.default_rng(24)
    T, B = 5, 3
    e = rng.standard_normal((T, B, m.joint_out.cols)).astype(np.float32)
    tok, ln, sc = oracle.decode(m, e, 3, 2)
    perm = [2, 0, 1]
    tok2, ln2, sc2 = oracle.decode(m, e[:, perm].copy(), 3, 2)
    assert np.array_equal(tok2, tok[perm]) and np.array_equal(ln2, ln[perm]) and np.array_equal(sc2, sc[perm])
    assert np.all(np.diff(sc, axis=1) <= 0)


def test_decode_lm_weights_zero_equals_no_lms():
    m = _tiny_model(25, V=5, lam=(0.0, 0.0))
    m2 = oracle.Model(m.pred, None, None, m.joint_out, 0.0, 0.0)
    rng = np.random.default_rng(25)
    e = rng.standard_normal((5, 2, m.joint_out.cols)).astype(np.float32)
    a = oracle.decode(m, e, 3, 2)
    b = oracle.decode(m2, e, 3, 2)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_golden_config0_decode_is_reproducible():
    """The stored config-0 beams (written by tests/golden/make_golden.py, which
    calls only the oracle) are what the GPU path is compared with."""
    path = os.path.join(GOLD, "cfg0_decode.txt")
    if not os.path.exists(path):
        pytest.skip("golden file not generated")
    from tests.golden import make_golden
    assert open(path).read() == make_golden.render()


def test_golden_config0_alsd_is_reproducible():
    """The stored finished lists of the alignment-length synchronous search (same script, oracle only)."""
    path = os.path.join(GOLD, "cfg0_alsd.txt")
    from tests.golden import make_golden
    assert open(path).read() == make_golden.render_alsd()


def test_quantizer_properties_over_random_boundaries():
    """Properties that Sec. 3.1's symmetric quantizer has at any boundary and width: codes stay in range, the map
    is odd except at the clipped end, monotone, idempotent on its own grid, and the residual inside the range is
    at most half a step."""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=60, deadline=None)
    @given(st.floats(0.05, 50.0), st.sampled_from([4, 8]), st.integers(0, 2 ** 31 - 1))
    def check(alpha, bits, seed):
        qmax = 127 if bits == 8 else 7
        inv = np.float32(qmax) / np.float32(alpha)
        step = float(np.float32(alpha) / np.float32(qmax))
        rng = np.random.default_rng(seed)
        x = (rng.standard_normal(400) * alpha).astype(np.float32)
        q = oracle.quant_sym(x, inv, bits).astype(np.int32)
        assert q.min() >= -qmax - 1 and q.max() <= qmax
        qn = oracle.quant_sym(-x, inv, bits).astype(np.int32)
        odd = (np.abs(q) <= qmax) & (np.abs(qn) <= qmax)
        assert np.array_equal(q[odd], -qn[odd])                         # rounding to even is an odd function
        order = np.argsort(x, kind="stable")
        assert np.all(np.diff(q[order]) >= 0)
        grid = (np.arange(-qmax, qmax + 1, dtype=np.float32) * np.float32(step)).astype(np.float32)
        back = oracle.quant_sym(grid, inv, bits).astype(np.int32)
        assert np.abs(back - np.arange(-qmax, qmax + 1)).max() <= (0 if bits == 4 else 1)   # fp32 alpha/qmax * qmax/alpha
        inside = np.abs(x) <= alpha
        assert np.all(np.abs(x[inside].astype(np.float64) - q[inside] * step) <= step / 2 * (1 + 1e-3) + 1e-7)

    check()


# ------------------------------------------------------------------ initial state of a layer

def test_lstm_layer_initial_state_closed_form_and_continuation():
    # zero weights and a given c0: c_1 = f c0 + i g exactly (h0 meets zero weights), so the layer started from
    # (h0, c0) must give c_t = f^t c0 + i g (1 - f^t)/(1 - f); and a layer run in two halves, the second started
    # from the first's final state, must equal the layer run in one piece (any weights).
    H, I, T, B = 5, 4, 9, 3
    rng = np.random.default_rng(41)
    b = rng.standard_normal(4 * H)
    L0 = oracle.Lstm(np.zeros((4 * H, I)), np.ones(4 * H), np.zeros((4 * H, H)), np.ones(4 * H), b, 0.3)
    x = rng.integers(-7, 8, (T, B, I)).astype(np.int8)
    h0 = rng.integers(-7, 8, (B, H)).astype(np.int8)
    c0 = rng.standard_normal((B, H)).astype(np.float32)
    _, _, _, c_all = oracle.lstm_layer(L0, x, h0=h0, c0=c0, want_c_all=True)
    b32 = b.astype(np.float32).astype(np.float64)
    sg = lambda v: 1 / (1 + np.exp(-v))
    i, f, g = sg(b32[:H]), sg(b32[H:2 * H]), np.tanh(b32[2 * H:3 * H])
    for t in range(1, T + 1):
        c = f ** t * c0.astype(np.float64) + i * g * (1 - f ** t) / (1 - f)
        assert np.allclose(c_all[t - 1], c, rtol=3e-6, atol=2e-7)
    L = _rand_lstm(rng, I, H)
    for reverse in (False, True):
        whole, hl, cl, _ = oracle.lstm_layer(L, x, reverse=reverse, h0=h0, c0=c0)
        first = x[T - 4:] if reverse else x[:5]
        second = x[:T - 4] if reverse else x[5:]
        a, ha, ca, _ = oracle.lstm_layer(L, first, reverse=reverse, h0=h0, c0=c0)
        bb, hb, cb, _ = oracle.lstm_layer(L, second, reverse=reverse, h0=ha, c0=ca)
        joined = np.concatenate([bb, a]) if reverse else np.concatenate([a, bb])
        assert np.array_equal(whole, joined) and np.array_equal(hl, hb) and np.array_equal(cl, cb)
        # the initial hidden codes matter too (non-zero recurrent weights), and None means zero
        other, _, _, _ = oracle.lstm_layer(L, x, reverse=reverse, h0=np.zeros_like(h0), c0=c0)
        assert not np.array_equal(other, whole)
        z1, _, _, _ = oracle.lstm_layer(L, x, reverse=reverse)
        z2, _, _, _ = oracle.lstm_layer(L, x, reverse=reverse, h0=np.zeros_like(h0), c0=np.zeros_like(c0))
        assert np.array_equal(z1, z2)


# ------------------------------------------------------------------ tie and selection margins (bookkeeping)

def _np_tie_distance(x, inv_s, qmax=7.0):
    t = (np.asarray(x, np.float32) * np.float32(inv_s)).astype(np.float64)
    d = np.abs(t - np.floor(t) - 0.5) * (7.0 / qmax)
    return np.where((t <= -qmax - 1.5) | (t >= qmax + 0.5), np.inf, d)


def test_tie_distance_hand_values():
    assert oracle.tie_distance(0.5, 7.0) == 0.0                       # 3.5: a tie
    assert oracle.tie_distance(np.float32(2.5) / np.float32(7), 7.0) < 3e-7
    assert oracle.tie_distance(1.0, 7.0) == 0.5                       # a grid value is as far from a tie as can be
    assert abs(oracle.tie_distance(0.3, 1.0) - 0.2) < 1e-7            # rounds to 0, 0.2 below the tie at 0.5
    assert abs(oracle.tie_distance(-1.2, 7.0) - 0.1) < 1e-5           # -8.4: 0.1 from the tie between -8 and the clamp at -8.5
    assert oracle.tie_distance(1.5, 7.0) == math.inf                  # 10.5: the clamp decides
    assert oracle.tie_distance(-1.3, 7.0) == math.inf                 # -9.1
    assert abs(oracle.tie_distance(1.071, 7.0) - 0.003) < 1e-5        # 7.497: the last tie before the clamp, at 7.5
    assert oracle.tie_distance(0.5, 127.0, 8) == 0.0                  # 63.5
    assert abs(oracle.tie_distance(0.5 + 0.25 / 127, 127.0, 8) - 0.25 * 7 / 127) < 1e-6   # in 4-bit code steps
    assert oracle.tie_distance(2.0, 127.0, 8) == math.inf


def test_layer_margin_is_the_smallest_tie_distance_of_each_utterance():
    rng = np.random.default_rng(42)
    I, H, T, B = 6, 8, 11, 4
    L = _rand_lstm(rng, I, H)
    x = rng.integers(-7, 8, (T, B, I)).astype(np.int8)
    um = np.full(B, np.inf)
    h_out, _, _, _ = oracle.lstm_layer(L, x, utt_margin=um)
    plain, _, _, _ = oracle.lstm_layer(L, x)
    assert np.array_equal(h_out, plain)
    hp, cp = np.zeros((B, H), np.int8), np.zeros((B, H), np.float32)
    want = np.full(B, np.inf)
    for t in range(T):
        hp, cp, dbg = oracle.lstm_step(L, x[t], hp, cp, debug=True)
        want = np.minimum(want, _np_tie_distance(dbg["h_real"], 7.0).min(axis=1))
    assert np.allclose(um, want, rtol=0, atol=1e-12) and np.all(um < 0.5) and len(set(um.tolist())) == B
    # an already lower entry stays (the argument is lowered, not overwritten)
    um2 = np.array([0.0, np.inf, np.inf, np.inf])
    oracle.lstm_layer(L, x, utt_margin=um2)
    assert um2[0] == 0.0 and np.allclose(um2[1:], want[1:], atol=1e-12)


def test_beam_step_gap_against_a_sort():
    rng = np.random.default_rng(43)
    B, W, V = 5, 3, 4
    score = rng.standard_normal((B, W)).astype(np.float32)
    fused = rng.standard_normal((B * W, V)).astype(np.float32)
    score[1, 1:] = -np.inf                       # 4 finite candidates: 3 picks + one left out
    score[2, 1:] = -np.inf; fused[2 * W, 2:] = -np.inf      # 2 finite candidates: nothing left out
    fused[3 * W, 0] = fused[3 * W, 1] = 50.0     # an exact tie among the picks
    for force in (False, True):
        par, tok, ns, gap = oracle.beam_step(score, fused, force_blank=force, want_gap=True)
        p2, t2, n2 = oracle.beam_step(score, fused, force_blank=force)
        assert np.array_equal(par, p2) and np.array_equal(tok, t2) and np.array_equal(ns, n2)
        for b in range(B):
            val = (score[b][:, None] + fused[b * W:(b + 1) * W]).astype(np.float32)
            if force:
                val[:, 1:] = -np.inf
            v = np.sort(val[np.isfinite(val)].astype(np.float64))[::-1][:W + 1]
            want = np.min(v[:-1] - v[1:]) if len(v) > 1 else np.inf
            assert gap[b] == want, (force, b)
    assert oracle.beam_step(score, fused, want_gap=True)[3][3] == 0.0


def test_decode_margins_on_a_path_that_can_be_recomputed():
    # margins are bookkeeping: same beams with and without them; and with one hypothesis and no labels per frame
    # (W = 1, max_sym = 0) the path is the start hypothesis at every frame, whose quantizer decisions can be
    # recomputed one by one: the start-symbol advance of each network and z at every frame.
    m = _tiny_model(44)
    rng = np.random.default_rng(45)
    T, B, J = 6, 3, m.joint_out.cols
    e = rng.standard_normal((T, B, J)).astype(np.float32)
    for W, ms in ((1, 0), (3, 2)):
        a = oracle.decode(m, e, W, ms, max_len=8)
        bq = oracle.decode(m, e, W, ms, max_len=8, margins=True)
        assert all(np.array_equal(x, y) for x, y in zip(a, bq[:3]))
        c = oracle.decode_alsd(m, e, W, 2)
        d = oracle.decode_alsd(m, e, W, 2, margins=True)
        assert all(np.array_equal(x, y) for x, y in zip(c, d[:3]))
        assert np.all(d[3] > 0) and np.all(d[3] < 0.5) and np.all(d[4] >= 0)
    _, _, _, qm, sm = oracle.decode(m, e, 1, 0, max_len=1, margins=True)
    start = np.inf
    for net in (m.pred, m.lm_src, m.lm_ext):
        xq = oracle.quant_sym4(net.embed[0][None], net.inv_s_e)
        H = net.layers[0].H
        _, _, dbg = oracle.lstm_step(net.layers[0], xq, np.zeros((1, H), np.int8), np.zeros((1, H), np.float32), debug=True)
        start = min(start, _np_tie_distance(dbg["h_real"], 7.0).min())
    p0 = oracle.net_run(m.pred, np.array([0], np.int32))
    for b in range(B):
        rows = np.array([t * B + b for t in range(T)], np.int32)
        _, z_real = oracle.joint_z(e.reshape(T * B, J), rows, np.repeat(p0, T, axis=0), 7.0)
        want = min(start, _np_tie_distance(z_real, 7.0).min())
        assert abs(qm[b] - want) < 1e-12, b
    assert np.all(np.isinf(sm))     # one candidate per selection: nothing is ranked against anything
    # a single frame: few z decisions, so for most utterances the start-symbol advance holds the smallest distance
    e1 = rng.standard_normal((1, 8, J)).astype(np.float32)
    _, _, _, qm1, _ = oracle.decode(m, e1, 1, 0, max_len=1, margins=True)
    _, _, _, qa1, _ = oracle.decode_alsd(m, e1, 1, 0, margins=True)
    assert np.all(qm1 <= start) and (qm1 == start).sum() >= 3 and np.array_equal(qm1, qa1)
    # a wider beam only adds decisions, and dead slots add none: the margin of utterance b does not depend on
    # what else is in the batch
    _, _, _, q3, s3 = oracle.decode(m, e, 3, 2, max_len=8, margins=True)
    assert np.all(q3 <= qm)
    _, _, _, q1, s1 = oracle.decode(m, np.ascontiguousarray(e[:, 1:2]), 3, 2, max_len=8, margins=True)
    assert q1[0] == q3[1] and s1[0] == s3[1]


# ------------------------------------------------------------------ reuse of cached hypotheses (Sec. 4.1)

def test_alsd_hypothesis_cache_changes_the_work_not_the_result():
    # the networks' states after a label sequence depend on the sequence alone: taking them over from a cache gives
    # the same finished lists bit for bit in every mode.  With a beam wide enough that nothing is pruned and 2 labels,
    # every label sequence of length 1..3 is extended at some iteration, many of them again and again (from the same
    # prefix one frame later): an unbounded cache advances the networks exactly once per distinct sequence,
    # 2 + 4 + 8 = 14 times, whatever the number of frames.
    m = _tiny_model(61)                      # V = 3: blank + 2 labels
    rng = np.random.default_rng(62)
    J = m.joint_out.cols
    for T in (1, 2, 4):
        e = rng.standard_normal((T, 2, J)).astype(np.float32)
        base = oracle.decode_alsd(m, e, 48, 3)
        outs = [oracle.decode_alsd_cached(m, e, 48, 3, mode) for mode in (0, 1, 2)]
        for o in outs:
            assert all(np.array_equal(a, b) for a, b in zip(o[:3], base))
        req0, done0 = outs[0][3], outs[0][4]
        assert np.array_equal(req0, done0)                       # no cache: every request is an advance
        assert np.all(outs[2][4] == 14), (T, outs[2][4])         # one advance per distinct sequence
        assert np.all(outs[1][3] == req0) and np.all(outs[2][3] == req0)
        assert np.all(outs[1][4] <= done0) and np.all(outs[2][4] <= outs[1][4])
        if T >= 2:
            assert np.all(req0 > 14) and np.all(outs[1][4] < req0)   # re-proposed sequences are found in the beam
    # a narrow beam on a longer utterance: still the same beams in every mode
    m2 = _tiny_model(63, V=5, rho=0.1)
    e = rng.standard_normal((9, 3, m2.joint_out.cols)).astype(np.float32)
    base = oracle.decode_alsd(m2, e, 4, 6)
    for mode in (0, 1, 2):
        o = oracle.decode_alsd_cached(m2, e, 4, 6, mode)
        assert all(np.array_equal(a, b) for a, b in zip(o[:3], base)) and np.all(o[4] <= o[3])
