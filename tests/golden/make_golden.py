"""Writes tests/golden/cfg0_decode.txt from the CPU oracle alone.

Run as ``python -m tests.golden.make_golden`` from the repository root.  The
file holds the beams the oracle decodes for the tiny configuration (1-layer
encoder H=64 over 32-dim features, T=20, B=2, vocabulary 16, joint 32, LMs
H=64, lambda_src 0.3, lambda_ext 0.5, beam 2, at most 4 labels per frame), at
the stated weight deviation 0.1 and at 0.6 (a variant that emits labels).  The
GPU decode is compared with it; nothing in it comes from the GPU.
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


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg0_decode.txt")
    with open(path, "w") as f:
        f.write(render())
    print(open(path).read())
