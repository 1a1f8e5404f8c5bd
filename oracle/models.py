"""Build oracle networks from float weights (test infrastructure only).

Takes any object with the attributes of the synthetic float description
(embed/layers/out, w_ih/w_hh/bias, w/bias) and quantizes it with the oracle's
own quantizers.  Imports nothing from the GPU package.
"""
from __future__ import annotations

import numpy as np

from . import Linear, Lstm, Model, Net, lstm_layer, linear, quant_sym, quant_sym4

S_H = np.float32(1.0) / np.float32(7.0)   # FIX +-1 step of hidden states and of z (Sec. 3.2)
S_H8 = np.float32(1.0) / np.float32(127.0)   # the same boundary at 8 bits


def act_scale(alpha, bits=4):
    """(step, 1/step) of a FIX activation quantizer with boundary alpha."""
    a = np.float32(alpha)
    qmax = np.float32(127.0 if bits == 8 else 7.0)
    return np.float32(a / qmax), np.float32(qmax / a)


def lstm_from_float(f, s_x, bits=4):
    if bits == 8:
        return Lstm.from_float(f.w_ih, f.w_hh, f.bias, s_x, S_H8, 127.0, bits=8)
    return Lstm.from_float(f.w_ih, f.w_hh, f.bias, s_x, S_H, 7.0)


def net_from_float(f, alpha_e, log_softmax, out_bits=4):
    s_e, _ = act_scale(alpha_e)
    layers = []
    for i, lf in enumerate(f.layers):
        layers.append(lstm_from_float(lf, s_e if i == 0 else S_H))
    mid = getattr(f, "mid", None)
    if mid is not None:   # bottleneck layer (Sec. 2): its output is quantized with boundary alpha_mid
        s_m, _ = act_scale(f.alpha_mid)
        return Net(f.embed, alpha_e, layers, Linear.from_float(f.out.w, f.out.bias, s_m), log_softmax,
                   mid=Linear.from_float(mid.w, mid.bias, S_H), alpha_mid=f.alpha_mid)
    out = Linear.from_float(f.out.w, f.out.bias, S_H, bits=out_bits)
    return Net(f.embed, alpha_e, layers, out, log_softmax)


def model_from_float(m, use_src=True, use_ext=True):
    if getattr(m, "mixed_precision", False):
        # Sec. 3.2: the RNN-T's linear layers at 8 bits (weights and their own input quantizer: z for the joint's
        # output layer; the prediction network's output layer reads the cell's 4-bit output codes, Sec. 3.4)
        pred = net_from_float(m.pred, m.alpha_e, False, out_bits=8)
        src = net_from_float(m.lm_src, m.alpha_e, True) if (use_src and m.lm_src is not None) else None
        ext = net_from_float(m.lm_ext, m.alpha_e, True) if (use_ext and m.lm_ext is not None) else None
        jout = Linear.from_float(m.joint_out.w, m.joint_out.bias, S_H8, bits=8)
        return Model(pred, src, ext, jout, m.lambda_src, m.lambda_ext, m.rho, blank=0, inv_s_z=127.0)
    pred = net_from_float(m.pred, m.alpha_e, False)
    src = net_from_float(m.lm_src, m.alpha_e, True) if (use_src and m.lm_src is not None) else None
    ext = net_from_float(m.lm_ext, m.alpha_e, True) if (use_ext and m.lm_ext is not None) else None
    jout = Linear.from_float(m.joint_out.w, m.joint_out.bias, S_H)
    return Model(pred, src, ext, jout, m.lambda_src, m.lambda_ext, m.rho, blank=0, inv_s_z=7.0)


def encoder_from_float(m):
    """List of layers, each a list of directions (Lstm), and the projection."""
    mixed = bool(getattr(m, "mixed_precision", False))
    s_x, _ = act_scale(m.alpha_x, 8 if mixed else 4)
    layers = []
    for li, dirs in enumerate(m.enc_layers):
        # mixed precision (Sec. 3.2): the first layer at 8 bits; the second layer reads its 8-bit hidden codes
        bits = 8 if (mixed and li == 0) else 4
        x_scale = s_x if li == 0 else (S_H8 if (mixed and li == 1) else S_H)
        layers.append([lstm_from_float(d, x_scale, bits) for d in dirs])
    s_top = S_H8 if (mixed and len(m.enc_layers) == 1) else S_H
    proj = Linear.from_float(m.enc_proj.w, m.enc_proj.bias, s_top, bits=8 if mixed else 4)
    return layers, proj


def encoder_forward(layers, proj, feats, alpha_x, utt_margin=None):
    """features [T,B,D] fp32 -> (codes of the last layer [T,B,dirs*H], e [T,B,J]).  The input quantizer has
    the width of the first layer.  utt_margin (float64 [B], optional) is lowered to the smallest tie distance of
    every hidden-state quantizer decision of each utterance."""
    bits = layers[0][0].bits
    _, inv_s_x = act_scale(alpha_x, bits)
    x = quant_sym(feats, inv_s_x, bits)
    T, B, _ = x.shape
    for dirs in layers:
        H = dirs[0].H
        out = np.zeros((T, B, H * len(dirs)), np.int8)
        for d, L in enumerate(dirs):
            lstm_layer(L, x, reverse=(d == 1), h_out=out, col_off=d * H, utt_margin=utt_margin)
        x = out
    e = linear(proj, x.reshape(T * B, -1)).reshape(T, B, -1)
    return x, e
