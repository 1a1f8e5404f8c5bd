"""Build oracle networks from float weights (test infrastructure only).

Takes any object with the attributes of the synthetic float description
(embed/layers/out, w_ih/w_hh/bias, w/bias) and quantizes it with the oracle's
own quantizers.  Imports nothing from the GPU package.
"""
from __future__ import annotations

import numpy as np

from . import Linear, Lstm, Model, Net, lstm_layer, linear, quant_sym4

S_H = np.float32(1.0) / np.float32(7.0)   # FIX +-1 step of hidden states and of z (Sec. 3.2)


def act_scale(alpha):
    """(step, 1/step) of a FIX activation quantizer with boundary alpha."""
    a = np.float32(alpha)
    return np.float32(a / np.float32(7.0)), np.float32(np.float32(7.0) / a)


def lstm_from_float(f, s_x):
    return Lstm.from_float(f.w_ih, f.w_hh, f.bias, s_x, S_H, 7.0)


def net_from_float(f, alpha_e, log_softmax):
    s_e, _ = act_scale(alpha_e)
    layers = []
    for i, lf in enumerate(f.layers):
        layers.append(lstm_from_float(lf, s_e if i == 0 else S_H))
    mid = getattr(f, "mid", None)
    if mid is not None:   # bottleneck layer (Sec. 2): its output is quantized with boundary alpha_mid
        s_m, _ = act_scale(f.alpha_mid)
        return Net(f.embed, alpha_e, layers, Linear.from_float(f.out.w, f.out.bias, s_m), log_softmax,
                   mid=Linear.from_float(mid.w, mid.bias, S_H), alpha_mid=f.alpha_mid)
    out = Linear.from_float(f.out.w, f.out.bias, S_H)
    return Net(f.embed, alpha_e, layers, out, log_softmax)


def model_from_float(m, use_src=True, use_ext=True):
    pred = net_from_float(m.pred, m.alpha_e, False)
    src = net_from_float(m.lm_src, m.alpha_e, True) if (use_src and m.lm_src is not None) else None
    ext = net_from_float(m.lm_ext, m.alpha_e, True) if (use_ext and m.lm_ext is not None) else None
    jout = Linear.from_float(m.joint_out.w, m.joint_out.bias, S_H)
    return Model(pred, src, ext, jout, m.lambda_src, m.lambda_ext, m.rho, blank=0, inv_s_z=7.0)


def encoder_from_float(m):
    """List of layers, each a list of directions (Lstm), and the projection."""
    s_x, _ = act_scale(m.alpha_x)
    layers = []
    for li, dirs in enumerate(m.enc_layers):
        layers.append([lstm_from_float(d, s_x if li == 0 else S_H) for d in dirs])
    proj = Linear.from_float(m.enc_proj.w, m.enc_proj.bias, S_H)
    return layers, proj


def encoder_forward(layers, proj, feats, alpha_x):
    """features [T,B,D] fp32 -> (codes of the last layer [T,B,dirs*H], e [T,B,J])."""
    _, inv_s_x = act_scale(alpha_x)
    x = quant_sym4(feats, inv_s_x)
    T, B, _ = x.shape
    for dirs in layers:
        H = dirs[0].H
        out = np.zeros((T, B, H * len(dirs)), np.int8)
        for d, L in enumerate(dirs):
            lstm_layer(L, x, reverse=(d == 1), h_out=out, col_off=d * H)
        x = out
    e = linear(proj, x.reshape(T * B, -1)).reshape(T, B, -1)
    return x, e
