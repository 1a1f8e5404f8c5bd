"""Device-side model assembly: float weights -> packed INT4 blobs via the C ABI.

Everything numeric happens in libqrnnt (qrnnt_pack_int4 quantizes and packs,
qrnnt_quantize_act quantizes embeddings and features); this module only moves
host arrays to the GPU and strings the ABI calls together.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import qrnnt as q

S_H = float(np.float32(1.0) / np.float32(7.0))     # FIX +-1 step (Sec. 3.2)
S_H8 = float(np.float32(1.0) / np.float32(127.0))  # the same boundary at 8 bits


def act_scale(alpha: float, bits: int = 4):
    a = np.float32(alpha)
    qmax = np.float32(127.0 if bits == 8 else 7.0)
    return float(np.float32(a / qmax)), float(np.float32(qmax / a))


def _pack(w, layout, bits):
    return q.pack_int8(w, layout) if bits == 8 else q.pack_int4(w, layout)


def _dev(a, device):
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def lstm_from_float(f, x_scale: float, device="cuda:0", bits: int = 4) -> q.Lstm:
    return q.Lstm(_pack(_dev(f.w_ih, device), q.LAYOUT_TILED_GATES, bits),
                  _pack(_dev(f.w_hh, device), q.LAYOUT_TILED_GATES, bits),
                  _dev(f.bias, device), x_scale, S_H8 if bits == 8 else S_H, 127.0 if bits == 8 else 7.0)


def net_from_float(f, alpha_e: float, log_softmax: bool, device="cuda:0", out_bits: int = 4) -> q.Net:
    """out_bits = 8: the output layer's weights at 8 bits (Sec. 3.2, the RNN-T's linear layers); its input
    stays the top layer's hidden codes, quantized once at the cell output (Sec. 3.4)."""
    s_e, inv_e = act_scale(alpha_e)
    embed_codes = q.quantize_act_rows(_dev(f.embed, device), inv_e)   # [V, act_pitch(E)]
    layers = [lstm_from_float(lf, s_e if i == 0 else S_H, device) for i, lf in enumerate(f.layers)]
    out = _pack(_dev(f.out.w, device), q.LAYOUT_TILED, out_bits)
    mid = getattr(f, "mid", None)
    if mid is not None:   # bottleneck between the LSTM stack and the output layer (Sec. 2, external LM)
        s_m, inv_m = act_scale(f.alpha_mid)
        return q.Net(embed_codes, layers, out, _dev(f.out.bias, device), S_H, log_softmax,
                     mid=q.pack_int4(_dev(mid.w, device), q.LAYOUT_TILED), mid_bias=_dev(mid.bias, device),
                     mid_scale=s_m, mid_inv_scale=inv_m)
    return q.Net(embed_codes, layers, out, _dev(f.out.bias, device), S_H, log_softmax)


def model_from_float(m, device="cuda:0", use_src=True, use_ext=True) -> q.Model:
    if getattr(m, "mixed_precision", False):
        # Sec. 3.2: the RNN-T's linear layers (prediction-network output, joint output) at 8 bits, z quantized
        # at 8 bits with them; the LMs stay 4-bit throughout
        pred = net_from_float(m.pred, m.alpha_e, False, device, out_bits=8)
        src = net_from_float(m.lm_src, m.alpha_e, True, device) if (use_src and m.lm_src is not None) else None
        ext = net_from_float(m.lm_ext, m.alpha_e, True, device) if (use_ext and m.lm_ext is not None) else None
        jout = q.pack_int8(_dev(m.joint_out.w, device), q.LAYOUT_TILED)
        return q.Model(pred, src, ext, jout, _dev(m.joint_out.bias, device), m.lambda_src, m.lambda_ext, m.rho,
                       z_scale=S_H8, z_inv_scale=127.0)
    pred = net_from_float(m.pred, m.alpha_e, False, device)
    src = net_from_float(m.lm_src, m.alpha_e, True, device) if (use_src and m.lm_src is not None) else None
    ext = net_from_float(m.lm_ext, m.alpha_e, True, device) if (use_ext and m.lm_ext is not None) else None
    jout = q.pack_int4(_dev(m.joint_out.w, device), q.LAYOUT_TILED)
    return q.Model(pred, src, ext, jout, _dev(m.joint_out.bias, device), m.lambda_src, m.lambda_ext, m.rho)


class Encoder:
    """Stack of (bi)directional quantized LSTM layers plus the projection to the joint."""

    def __init__(self, m, device="cuda:0"):
        # mixed precision (Sec. 3.2): first layer and the projection at 8 bits; the second layer reads the first
        # layer's 8-bit hidden codes (one quantizer per cell output, Sec. 3.4)
        self.mixed = bool(getattr(m, "mixed_precision", False))
        self.s_x, self.inv_s_x = act_scale(m.alpha_x, 8 if self.mixed else 4)
        self.layers: List[List[q.Lstm]] = []
        for li, dirs in enumerate(m.enc_layers):
            bits = 8 if (self.mixed and li == 0) else 4
            x_scale = self.s_x if li == 0 else (S_H8 if (self.mixed and li == 1) else S_H)
            self.layers.append([lstm_from_float(d, x_scale, device, bits) for d in dirs])
        self.proj = _pack(_dev(m.enc_proj.w, device), q.LAYOUT_TILED, 8 if self.mixed else 4)
        self.proj_a_scale = S_H8 if (self.mixed and len(m.enc_layers) == 1) else S_H
        self.proj_bias = _dev(m.enc_proj.bias, device)
        self._ws: Optional[torch.Tensor] = None
        # bounded-wait flags of the persistent recurrence, one per layer-direction, as the last forward left them
        self._flags = torch.zeros(sum(len(d) for d in self.layers), dtype=torch.int32, device=device)

    def workspace(self, T: int, B: int, device) -> torch.Tensor:
        need = max(sum(q.lstm_layer_workspace(L, T, B) for L in dirs) for dirs in self.layers)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=device)
        return self._ws

    def forward(self, feats: torch.Tensor):
        """feats [T,B,D] fp32 on the device -> (codes [T,B,dirs*H], e [T,B,J] fp32)."""
        T, B, _ = feats.shape
        ws = self.workspace(T, B, feats.device)
        x = q.quantize_act_rows(feats, self.inv_s_x, 8 if self.mixed else 4)   # [T, B, act_pitch(D)]
        k = 0
        for dirs in self.layers:
            H = dirs[0].H
            out = torch.empty((T, B, H * len(dirs)), dtype=torch.int8, device=feats.device)
            ends = []   # where each direction's workspace ends: its flag sits 256 bytes before
            for L in dirs:
                ends.append((ends[-1] if ends else 0) + q.lstm_layer_workspace(L, T, B))
            if len(dirs) == 2:
                q.bilstm_layer(dirs[0], dirs[1], x, h_out=out, workspace=ws)
            else:
                q.lstm_layer(dirs[0], x, h_out=out, col_off=0, workspace=ws)
            for end in ends:   # the workspace is reused by the next layer: keep the flag (4 bytes, device to device)
                self._flags[k:k + 1].copy_(ws[end - 256:end - 252].view(torch.int32))
                k += 1
            x = out
        e = q.linear(self.proj, self.proj_bias, self.proj_a_scale, x.reshape(T * B, -1)).reshape(T, B, -1)
        return x, e

    def check(self) -> None:
        """Raises if a bounded wait of the persistent recurrence ran out in the last forward (its outputs are then
        invalid).  One small device-to-host copy: call it outside timed regions."""
        flags = self._flags.cpu().tolist()
        if any(flags):
            raise RuntimeError(f"persistent recurrence: a bounded wait ran out (flags per layer-direction: {flags}); "
                               "was other work running on the device?")
