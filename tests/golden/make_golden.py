"""Writes tests/golden/cfg0_decode.txt and tests/golden/cfg0_alsd.txt from the CPU oracle alone.

Run as ``python -m tests.golden.make_golden`` from the repository root.  The
file holds the beams the oracle decodes for the tiny configuration (1-layer
encoder H=64 over 32-dim features, T=20, B=2, vocabulary 16, joint 32, LMs
H=64, lambda_src 0.3, lambda_ext 0.5, beam 2, at most 4 labels per frame), at
the stated weight deviation 0.1 and at 0.6 (a variant that emits labels).  The
GPU decode is compared with it; nothing in it comes from the GPU.
cfg0_alsd.txt holds the finished lists of the alignment-length synchronous search
with recombination on the same inputs (beam 4, at most 12 labels per utterance).
"""
import os

import numpy as np

import oracle
from oracle import models
from paper_2206_07882_amd import synth

T, B = 20, 2
STDS = (0.1, 0.6)


def decode_cfg0(std):
    m = synth.make_model(0, weight_std=std)
    layers, proj = models.encoder_from_float(m)
    feats = synth.features(0, T, B, m.feat_dim)
    _, e = models.encoder_forward(layers, proj, feats, m.alpha_x)
    M = models.model_from_float(m)
    return oracle.decode(M, e, m.beam, m.max_sym)


def render():
    lines = ["# config 0 decode by the CPU oracle: std, utterance, rank, score, labels"]
    for std in STDS:
        tok, ln, sc = decode_cfg0(std)
        for b in range(B):
            for w in range(tok.shape[1]):
                labs = " ".join(str(int(t)) for t in tok[b, w, :max(ln[b, w], 0)])
                lines.append(f"{std} {b} {w} {float(sc[b, w]):.4f} | {labs}")
    return "\n".join(lines) + "\n"


ALSD_W, ALSD_UMAX = 4, 12


def alsd_cfg0(std):
    m = synth.make_model(0, weight_std=std)
    layers, proj = models.encoder_from_float(m)
    feats = synth.features(0, T, B, m.feat_dim)
    _, e = models.encoder_forward(layers, proj, feats, m.alpha_x)
    return oracle.decode_alsd(models.model_from_float(m), e, ALSD_W, ALSD_UMAX)


def render_alsd():
    lines = ["# config 0, alignment-length synchronous search by the CPU oracle: std, utterance, rank, score, labels"]
    for std in STDS:
        tok, ln, sc = alsd_cfg0(std)
        for b in range(B):
            for w in range(tok.shape[1]):
                if ln[b, w] < 0:
                    continue
                labs = " ".join(str(int(t)) for t in tok[b, w, :ln[b, w]])
                lines.append(f"{std} {b} {w} {float(sc[b, w]):.4f} | {labs}")
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    for name, text in (("cfg0_decode.txt", render()), ("cfg0_alsd.txt", render_alsd())):
        with open(os.path.join(here, name), "w") as f:
            f.write(text)
        print(text)
