"""Seeded synthetic inputs with the shapes of the measured configurations.

This module draws random numbers and nothing else: it holds none of the
method's arithmetic (no quantizer, no scale, no matmul), so the CPU oracle's
tests and the GPU path can both take their inputs from it without sharing any
computation.  Everything is float32/int32 numpy on the host; the seed of
configuration ``i`` is ``20220607 + i``.

Recipe (stands in for trained weights and speech features, which are not
available): features ~ N(0,1); LSTM and linear weights ~ N(0, 1/sqrt(fan_in))
(config 0: N(0, 0.1) as its description states); biases ~ N(0, 0.1);
embeddings ~ N(0, 0.5).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

BASE_SEED = 20220607


@dataclass
class LstmF:
    w_ih: np.ndarray   # [4H, I] gate rows i,f,g,o
    w_hh: np.ndarray   # [4H, H]
    bias: np.ndarray   # [4H]


@dataclass
class LinearF:
    w: np.ndarray      # [rows, cols]
    bias: np.ndarray   # [rows]


@dataclass
class NetF:
    embed: np.ndarray          # [V, E]
    layers: List[LstmF]
    out: LinearF               # pred: [J, H]; LM: [V, H] ([V, M] behind a bottleneck)
    mid: Optional[LinearF] = None   # bottleneck [M, H] of the external LM (Sec. 2)
    alpha_mid: float = 4.0     # boundary of the quantizer on the bottleneck's output


@dataclass
class ModelF:
    """Float description of one configuration (None where a part is absent)."""
    name: str
    V: int
    J: int
    enc_layers: List[List[LstmF]] = field(default_factory=list)   # [layer][direction]
    enc_proj: Optional[LinearF] = None
    pred: Optional[NetF] = None
    lm_src: Optional[NetF] = None
    lm_ext: Optional[NetF] = None
    joint_out: Optional[LinearF] = None
    feat_dim: int = 0
    alpha_x: float = 4.0       # clipping boundary of the input features (4 sigma)
    alpha_e: float = 1.25      # boundary of the embedding quantizers
    lambda_src: float = 0.3
    lambda_ext: float = 0.5
    rho: float = 0.0
    beam: int = 16
    max_sym: int = 4
    mixed_precision: bool = False   # Sec. 3.2: first encoder layer and the RNN-T's linear layers at 8 bits


def _lstm(rng, I, H, std_ih=None, std_hh=None):
    si = std_ih if std_ih is not None else 1.0 / np.sqrt(I)
    sh = std_hh if std_hh is not None else 1.0 / np.sqrt(H)
    return LstmF(
        w_ih=(rng.standard_normal((4 * H, I)) * si).astype(np.float32),
        w_hh=(rng.standard_normal((4 * H, H)) * sh).astype(np.float32),
        bias=(rng.standard_normal(4 * H) * 0.1).astype(np.float32),
    )


def _linear(rng, rows, cols, std=None):
    s = std if std is not None else 1.0 / np.sqrt(cols)
    return LinearF(w=(rng.standard_normal((rows, cols)) * s).astype(np.float32),
                   bias=(rng.standard_normal(rows) * 0.1).astype(np.float32))


def _net(rng, V, E, hidden, n_layers, out_rows, std=None, mid=None):
    """mid: width of a bottleneck layer between the LSTM stack and the output layer."""
    embed = (rng.standard_normal((V, E)) * 0.5).astype(np.float32)
    layers = []
    for l in range(n_layers):
        layers.append(_lstm(rng, E if l == 0 else hidden, hidden, std, std))
    if mid is None:
        return NetF(embed=embed, layers=layers, out=_linear(rng, out_rows, hidden, std))
    # the bottleneck's outputs are sums of `hidden` terms of unit-variance scale: boundary at 4 sigma
    return NetF(embed=embed, layers=layers, mid=_linear(rng, mid, hidden, std), out=_linear(rng, out_rows, mid, std),
                alpha_mid=4.0 * 0.45)


def make_model(config: int, *, enc_layers: Optional[int] = None, weight_std: float = 0.1, mixed: bool = False) -> ModelF:
    """Float weights of configuration 0..4.  Configurations 1-3 describe parts
    of the full network; each returns only the parts it names.  ``weight_std``
    applies to configuration 0 only (its description fixes 0.1; larger values
    give a tiny network that actually emits labels, for search tests).
    Configuration 5 is the full network with the layer shapes of the paper's
    Sec. 2.  ``mixed`` marks the model for the precision map of Sec. 3.2 (first
    encoder layer and the RNN-T's linear layers at 8 bits); the float weights
    are the same either way."""
    if mixed:   # same float weights, quantized with the precision map of Sec. 3.2
        m = make_model(config, enc_layers=enc_layers, weight_std=weight_std)
        m.mixed_precision = True
        m.name += "-mixed"
        return m
    rng = np.random.default_rng(BASE_SEED + config)
    if config == 0:
        V, J, H = 16, 32, 64
        sd = weight_std
        m = ModelF(name="cfg0-tiny", V=V, J=J, feat_dim=32, beam=2, max_sym=4)
        m.enc_layers = [[_lstm(rng, 32, H, sd, sd)]]
        m.enc_proj = _linear(rng, J, H, sd)
        m.pred = _net(rng, V, H, H, 1, J, sd)
        m.lm_src = _net(rng, V, H, H, 1, V, sd)
        m.lm_ext = _net(rng, V, H, H, 1, V, sd)
        m.joint_out = _linear(rng, V, J, sd)
        return m
    V, J = 46, 256
    if config == 5:
        # The shapes of Sec. 2 (all 4-bit here): 340 input features, prediction network and source LM 1 x 768
        # cells over a 10-dimensional embedding, external LM 2 x 2048 cells over a 15-dimensional embedding +
        # bottleneck 256 (the parameter counts of Sec. 2, 2.6 M and 51.0 M, imply those embedding sizes), and
        # the fusion weights of Eq. 1 (mu = 0.7 on the external LM, lambda = 0.5 on the source LM, rho = 0.2
        # per label).
        m = ModelF(name="cfg5-paper-shapes", V=V, J=J, feat_dim=340, lambda_src=0.5, lambda_ext=0.7, rho=0.2)
        nl = 6 if enc_layers is None else enc_layers
        for l in range(nl):
            I = 340 if l == 0 else 1280
            m.enc_layers.append([_lstm(rng, I, 640), _lstm(rng, I, 640)])
        m.enc_proj = _linear(rng, J, 1280)
        m.pred = _net(rng, V, 10, 768, 1, J)
        m.joint_out = _linear(rng, V, J)
        m.lm_src = _net(rng, V, 10, 768, 1, V)
        m.lm_ext = _net(rng, V, 15, 2048, 2, V, mid=256)
        return m
    m = ModelF(name=f"cfg{config}", V=V, J=J, feat_dim=240)
    if config in (1, 4):
        nl = 6 if enc_layers is None else enc_layers
        for l in range(nl):
            I = 240 if l == 0 else 1280
            m.enc_layers.append([_lstm(rng, I, 640), _lstm(rng, I, 640)])
        m.enc_proj = _linear(rng, J, 1280)
    if config in (2, 4):
        m.pred = _net(rng, V, 768, 768, 1, J)
        m.joint_out = _linear(rng, V, J)
        if config == 2:
            m.enc_proj = _linear(rng, J, 1280)
    if config in (3, 4):
        m.lm_src = _net(rng, V, 256, 1024, 2, V)
        m.lm_ext = _net(rng, V, 256, 1024, 2, V)
        if config == 3:
            m.joint_out = _linear(rng, V, J)
    return m


def features(config: int, T: int, B: int, dim: int) -> np.ndarray:
    """Acoustic features [T, B, dim] ~ N(0,1)."""
    rng = np.random.default_rng(BASE_SEED + config + 1000)
    return rng.standard_normal((T, B, dim)).astype(np.float32)


def codes(seed: int, shape, lo: int = -7, hi: int = 7) -> np.ndarray:
    """Uniform integer codes in [lo, hi] as int8."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=shape).astype(np.int8)


def normal(seed: int, shape, std: float = 1.0) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape) * std).astype(np.float32)


def token_ids(seed: int, shape, V: int) -> np.ndarray:
    """Label ids uniform over 1..V-1 (0 is the blank / start symbol)."""
    rng = np.random.default_rng(seed)
    return rng.integers(1, V, size=shape).astype(np.int32)


def parent_perm(seed: int, B: int, W: int) -> np.ndarray:
    """For each utterance a random parent slot per hypothesis, as global slot
    indices b*W + w (parents never cross utterances)."""
    rng = np.random.default_rng(seed)
    p = rng.integers(0, W, size=(B, W)) + (np.arange(B)[:, None] * W)
    return p.reshape(-1).astype(np.int32)


def log_probs(seed: int, N: int, V: int) -> np.ndarray:
    """Rows that are logs of a random point of the simplex (a Dirichlet(1) draw),
    used as stand-ins for language-model outputs in teacher-forced tests."""
    rng = np.random.default_rng(seed)
    return np.log(rng.dirichlet(np.ones(V), size=N)).astype(np.float32)
