"""Configurations 2 and 3 as scripted step sequences at their full size (64 utterances x beam 16 =
1024 hypotheses, full layer widths), driven through the per-kernel entry points of the C ABI with the
state carried on the GPU.  Every step is checked teacher-forced on every hypothesis: the oracle
recomputes the step from the GPU's own state of the step before (hypotheses are independent), so a
rounding tie cannot travel.
Configuration 2: prediction network + joint under a seeded emission script (blanks advance a
hypothesis' frame, labels advance its prediction network; every step all hypotheses run the joint).
Configuration 3: both LMs step on random labels and parents, then the joint with the fusion of Eq. 1
and the top-16 selection per utterance.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import models as omodels
from paper_2206_07882_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
S_H = float(np.float32(1.0) / np.float32(7.0))
B, W, V, J = 64, 16, 46, 256
N = B * W


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def _codes_close(got, ref, h_real, what):
    """Equal, or one code apart where the fp64 value sits on a rounding tie."""
    diff = got.astype(np.int32) - ref
    bad = np.nonzero(diff)
    assert len(bad[0]) <= max(1, got.size // 10000), what
    if len(bad[0]) == 0:
        return
    t = h_real[bad] * 7.0
    assert np.all(np.abs(diff[bad]) == 1) and np.all(np.abs(np.abs(t - np.floor(t)) - 0.5) < 1e-4), what


def _rel(got, ref, what, tol=1e-5):
    assert np.all(np.abs(got - ref) <= tol * np.abs(ref) + 1e-6), what


def test_config2_prediction_and_joint_under_an_emission_script(gpu_lib):
    from paper_2206_07882_amd import model as gmodel
    q = gpu_lib
    m = synth.make_model(2)
    T_enc, steps = 500, 6
    rng = np.random.default_rng(20220609)
    enc_codes = synth.codes(901, (T_enc, B, 1280), -7, 7)
    # the script: a label (uniform over 1..45) with probability 1/3, else blank
    script = np.where(rng.random((steps, N)) < 1.0 / 3.0, rng.integers(1, V, (steps, N)), 0).astype(np.int32)
    rows = np.arange(N)                              # every hypothesis is recomputed by the oracle
    utt = (np.arange(N) // W).astype(np.int32)

    Gp = gmodel.net_from_float(m.pred, m.alpha_e, False, DEV)
    Op = omodels.net_from_float(m.pred, m.alpha_e, False)
    proj_g = q.pack_int4(dev(m.enc_proj.w), q.LAYOUT_TILED)
    proj_o = oracle.Linear.from_float(m.enc_proj.w, m.enc_proj.bias, S_H)
    jout_g = q.pack_int4(dev(m.joint_out.w), q.LAYOUT_TILED)
    jout_o = oracle.Linear.from_float(m.joint_out.w, m.joint_out.bias, S_H)
    jb = dev(m.joint_out.bias)
    e_g = q.linear(proj_g, dev(m.enc_proj.bias), S_H, dev(enc_codes.reshape(T_enc * B, 1280)))   # [T*B, J]
    embed_codes = host(Gp.embed_codes)
    assert np.array_equal(embed_codes, oracle.quant_sym4(m.pred.embed, Op.inv_s_e))

    L_g, L_o = Gp.layers[0], Op.layers[0]
    h = torch.zeros((N, L_g.H), dtype=torch.int8, device=DEV)
    c = torch.zeros((N, L_g.H), dtype=torch.float32, device=DEV)
    frame = np.zeros(N, np.int32)
    tok = np.zeros(N, np.int32)                      # every hypothesis first consumes the start symbol
    active = np.ones(N, np.uint8)
    n_label_steps = 0
    for s in range(steps + 1):
        # prediction network: the hypotheses whose last action was a label advance, the others keep their state
        hn, cn = q.lstm_step(L_g, Gp.embed_codes, h, c, x_row=dev(tok), active=dev(active))
        hr, cr, dbg = oracle.lstm_step(L_o, embed_codes[tok[rows]], host(h)[rows], host(c)[rows], active=active[rows],
                                       debug=True)
        act = active[rows].astype(bool)
        _rel(host(cn)[rows], cr, f"step {s}: c")
        _codes_close(host(hn)[rows][act], hr[act], dbg["h_real"][act], f"step {s}: h codes")
        assert np.array_equal(host(hn)[rows][~act], host(h)[rows][~act])
        n_label_steps += int(act.sum())
        h, c = hn, cn
        p_g = q.linear(Gp.out, Gp.out_bias, S_H, h)
        _rel(host(p_g)[rows], oracle.linear(Op.out, host(h)[rows]), f"step {s}: p")
        # joint for every hypothesis at its own frame
        frow = (frame * B + utt).astype(np.int32)
        fused, lp, zq = q.joint_fuse(e_g, dev(frow), p_g, jout_g, jb, None, None, 0.0, 0.0, want_lp=True, want_zq=True)
        e_rows = oracle.linear(proj_o, enc_codes.reshape(T_enc * B, 1280)[frow[rows]])
        _rel(host(e_g)[frow[rows]], e_rows, f"step {s}: e")
        _, lp_r, fused_r = oracle.joint_fuse(e_rows, np.arange(len(rows), dtype=np.int32), host(p_g)[rows], jout_o,
                                             None, None, 0.0, 0.0)
        assert np.abs(host(lp)[rows] - lp_r).max() < 1e-3 and np.abs(host(fused)[rows] - fused_r).max() < 1e-3
        assert np.abs(np.exp(host(lp).astype(np.float64)).sum(axis=1) - 1.0).max() < 1e-4    # every row, not only the sample
        if s == steps:
            break
        tok = script[s]
        active = (tok != 0).astype(np.uint8)
        frame = frame + (tok == 0)
    assert n_label_steps > len(rows)      # the script did advance sampled hypotheses beyond the start symbol


def test_config3_dual_lm_step_fusion_and_selection(gpu_lib):
    from paper_2206_07882_amd import model as gmodel
    q = gpu_lib
    m = synth.make_model(3)
    steps = 4
    lam_src, lam_ext = 0.3, 0.5
    rng = np.random.default_rng(20220610)
    rows = np.arange(N)                              # every hypothesis is recomputed by the oracle
    nets_g = [gmodel.net_from_float(f, m.alpha_e, True, DEV) for f in (m.lm_src, m.lm_ext)]
    nets_o = [omodels.net_from_float(f, m.alpha_e, True) for f in (m.lm_src, m.lm_ext)]
    jout_g = q.pack_int4(dev(m.joint_out.w), q.LAYOUT_TILED)
    jout_o = oracle.Linear.from_float(m.joint_out.w, m.joint_out.bias, S_H)
    jb = dev(m.joint_out.bias)
    e = synth.normal(911, (B, J), 1.0)               # one encoder frame per utterance
    p = synth.normal(912, (N, J), 1.0)               # a fixed prediction-network output per hypothesis
    frow = (np.arange(N) // W).astype(np.int32)
    embeds = [host(g.embed_codes) for g in nets_g]
    state = [[(torch.zeros((N, L.H), dtype=torch.int8, device=DEV), torch.zeros((N, L.H), dtype=torch.float32, device=DEV))
              for L in g.layers] for g in nets_g]
    score = synth.normal(913, (B, W), 1.0)
    for s in range(steps):
        tok = synth.token_ids(920 + s, (N,), V)
        parent = synth.parent_perm(930 + s, B, W) if s > 0 else np.arange(N, dtype=np.int32)
        lps = []
        for k, (g, o) in enumerate(zip(nets_g, nets_o)):
            x_codes, x_row = g.embed_codes, dev(tok)
            x_ref = embeds[k][tok[rows]]
            new_state = []
            for l, (L_g, L_o) in enumerate(zip(g.layers, o.layers)):
                hp, cp = state[k][l]
                hn, cn = q.lstm_step(L_g, x_codes, hp, cp, x_row=x_row, parent=dev(parent))
                hr, cr, dbg = oracle.lstm_step(L_o, x_ref, host(hp)[parent[rows]], host(cp)[parent[rows]], debug=True)
                _rel(host(cn)[rows], cr, f"step {s} net {k} layer {l}: c")
                _codes_close(host(hn)[rows], hr, dbg["h_real"], f"step {s} net {k} layer {l}: h codes")
                new_state.append((hn, cn))
                x_codes, x_row, x_ref = hn, None, host(hn)[rows]
            state[k] = new_state
            lp = q.linear(g.out, g.out_bias, S_H, x_codes, log_softmax=True)
            lp_r = oracle.log_softmax(oracle.linear(o.out, host(x_codes)[rows]))
            assert np.abs(host(lp)[rows] - lp_r).max() < 1e-3, f"step {s} net {k}: log-probs"
            lps.append(lp)
        fused, _, _ = q.joint_fuse(dev(e), dev(frow), dev(p), jout_g, jb, lps[0], lps[1], lam_src, lam_ext)
        _, _, fused_r = oracle.joint_fuse(e[frow[rows]], np.arange(len(rows), dtype=np.int32), p[rows], jout_o,
                                          host(lps[0])[rows], host(lps[1])[rows], lam_src, lam_ext)
        assert np.abs(host(fused)[rows] - fused_r).max() < 1e-3, f"step {s}: fused"
        # top-16 of 736 per utterance: exact against the oracle on the GPU's own fused scores
        par_g, tok_g, ns_g = q.beam_step(dev(score), fused)
        par_r, tok_r, ns_r = oracle.beam_step(score, host(fused))
        assert np.array_equal(host(par_g), par_r) and np.array_equal(host(tok_g), tok_r) and np.array_equal(host(ns_g), ns_r)
        score = ns_r
