#!/usr/bin/env python3
"""Benchmark of the INT4 RNN-T hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input:
feature quantization, 6 bidirectional INT4 LSTM layers (input-projection GEMM +
recurrence), the projection to the joint, and the full on-device beam search
with density-ratio fusion (beam 16, at most 4 labels per frame), i.e. the
end-to-end configuration: 64 utterances x 1000 frames of 40 ms = 2560 s of audio.
All inputs are resident in HBM before the timed region.  The printed value is the
real-time factor (processing time / audio duration, lower is better).

Besides the end-to-end figure the JSON line carries
  roofline      the dominant kernel (the fused LSTM step at 1024 hypotheses, as
                launched in one decoding round: prediction net, 2 x LM layer 1,
                2 x LM layer 2) against the dense int8 MFMA peak, timed with HIP
                events on the launch stream;
  extra         input-projection GEMM TOP/s, beam-16 (N=16) step GB/s, encoder
                and decoder split;
  cpu_baseline  the CPU oracle timed on this host on a bounded slice.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8, TOP/s (published)
HBM_PEAK_GBPS = 8000.0
FRAME_SEC = 0.04


def step_ops(I, H, N):
    return 2.0 * 4 * H * (I + H) * N


def step_bytes(I, H, N):
    """Algorithmic bytes of one fused LSTM step: packed weights, two scale vectors
    and the bias, input and hidden codes in (int8 containers), fp32 cell state in
    and out, hidden codes out, parent indices."""
    return 4 * H * (I + H) / 2 + 4 * H * 12 + N * (I + H) + 2 * N * H * 4 + N * H + 4 * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--leg", default="all", choices=["all", "e2e", "kernels"],
                    help="e2e: only the end-to-end step; kernels: only the per-kernel legs")
    ap.add_argument("--B", type=int, default=64)
    ap.add_argument("--T", type=int, default=1000)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (utterances would shard with no "
              "collective; see DESIGN.md). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2206_07882_amd import model as gmodel
    from paper_2206_07882_amd import qrnnt as q
    from paper_2206_07882_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    q.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    B, T, W, MAX_SYM = args.B, args.T, 16, 4
    m = synth.make_model(4)
    enc = gmodel.Encoder(m, dev)
    G = gmodel.model_from_float(m, dev)
    result = {"metric": "end_to_end_rtf_beam16", "unit": "s/s", "n_gpus": 1, "steps": args.steps,
              "warmup": args.warmup, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
              "dtype": "int4 codes on int8 MFMA, int32 accumulate, fp32 cell", "data": "synthetic",
              "config": {"workload": f"config 4: 6x bi-LSTM-640 encoder + pred-768 + 2 LMs 2x1024 + joint-256/46, "
                                     f"beam {W}, max {MAX_SYM} labels/frame, B={B} x T={T} frames ({B * T * FRAME_SEC:.0f} s audio)"}}
    extra = {}

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def timed(fn, iters, warm=2):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e-3   # seconds per call

    # ---------------------------------------------------------------- end to end
    if args.leg in ("all", "e2e"):
        feats = torch.from_numpy(synth.features(4, T, B, m.feat_dim)).to(dev)
        ws_dec = torch.empty(q.decode_workspace(G, T, B, W, MAX_SYM), dtype=torch.uint8, device=dev)
        enc.workspace(T, B, dev)

        def one_step():
            _, e = enc.forward(feats)
            return q.decode(G, e, W, MAX_SYM, max_len=T * MAX_SYM, workspace=ws_dec)

        for _ in range(args.warmup):
            one_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            out = one_step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        sec = (t1 - t0) / args.steps
        audio = B * T * FRAME_SEC
        result["value"] = sec / audio
        result["ms_per_step"] = sec * 1e3
        # split (separately timed, one pass each)
        t_enc = timed(lambda: enc.forward(feats), 1, warm=0)
        _, e = enc.forward(feats)
        t_dec = timed(lambda: q.decode(G, e, W, MAX_SYM, max_len=T * MAX_SYM, workspace=ws_dec), 1, warm=0)
        extra["encoder_ms"] = t_enc * 1e3
        extra["decoder_ms"] = t_dec * 1e3
        extra["audio_seconds_per_second"] = audio / sec
        lens = out[1].cpu().numpy()
        extra["mean_labels_best_hyp"] = float(lens[:, 0].mean())
        del feats, ws_dec, e, out

    # ---------------------------------------------------------------- kernel legs
    if args.leg in ("all", "kernels"):
        N = 1024
        rng = np.random.default_rng(7)

        def mk_state(n, H):
            return (torch.from_numpy(synth.codes(1, (n, H))).to(dev), torch.from_numpy(synth.normal(2, (n, H), 0.5)).to(dev))

        # the five LSTM launches of one decoding round at N = 64 x 16 hypotheses
        nets = [(G.pred, 0), (G.lm_src, 0), (G.lm_ext, 0), (G.lm_src, 1), (G.lm_ext, 1)]
        tok = torch.from_numpy(synth.token_ids(3, (N,), m.V)).to(dev)
        parent = torch.from_numpy(synth.parent_perm(4, N // W, W)).to(dev)
        calls, ops, byt = [], 0.0, 0.0
        for net, l in nets:
            L = net.layers[l]
            hp, cp = mk_state(N, L.H)
            if l == 0:
                x, xr = net.embed_codes, tok
            else:
                x, xr = torch.from_numpy(synth.codes(5, (N, L.I))).to(dev), None
            hn = torch.empty((N, L.H), dtype=torch.int8, device=dev)
            cn = torch.empty((N, L.H), dtype=torch.float32, device=dev)
            calls.append((L, x, xr, hp, cp, hn, cn))
            ops += step_ops(L.I, L.H, N)
            byt += step_bytes(L.I, L.H, N)

        def round_steps():
            for (L, x, xr, hp, cp, hn, cn) in calls:
                q.lstm_step_into(L, x, hp, cp, hn, cn, N, x_row=xr, parent=parent)

        t_round = timed(round_steps, 50, warm=5)
        per_launch = t_round / len(calls)
        ach = ops / len(calls) / per_launch / 1e12
        result["roofline"] = {"bound": "mfma", "kernel": "lstm_step_kernel (fused W4A4 LSTM step), N=1024 decode-round mix",
                              "achieved": ach, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                              "frac": ach / INT8_MFMA_PEAK_TOPS, "traffic": None,
                              "avg_launch_us": per_launch * 1e6, "ops_per_launch": ops / len(calls),
                              "algorithmic_bytes_per_launch": byt / len(calls),
                              "achieved_GBps": byt / len(calls) / per_launch / 1e9}

        # beam-16 regime (one utterance): weight streaming, reported against HBM
        N16 = 16
        parent16 = torch.from_numpy(synth.parent_perm(6, 1, W)).to(dev)
        calls16, byt16, ops16 = [], 0.0, 0.0
        for net, l in nets:
            L = net.layers[l]
            hp, cp = mk_state(N16, L.H)
            if l == 0:
                x, xr = net.embed_codes, tok[:N16].contiguous()
            else:
                x, xr = torch.from_numpy(synth.codes(5, (N16, L.I))).to(dev), None
            hn = torch.empty((N16, L.H), dtype=torch.int8, device=dev)
            cn = torch.empty((N16, L.H), dtype=torch.float32, device=dev)
            calls16.append((L, x, xr, hp, cp, hn, cn))
            byt16 += step_bytes(L.I, L.H, N16)
            ops16 += step_ops(L.I, L.H, N16)

        def round16():
            for (L, x, xr, hp, cp, hn, cn) in calls16:
                q.lstm_step_into(L, x, hp, cp, hn, cn, N16, x_row=xr, parent=parent16)

        t16 = timed(round16, 200, warm=10)
        extra["step_n16_warm"] = {"us_per_launch": t16 / 5 * 1e6, "GBps": byt16 / t16 / 1e9,
                                  "frac_hbm": byt16 / t16 / 1e9 / HBM_PEAK_GBPS, "bytes_per_round": byt16}

        # input-projection GEMM, encoder layers 1-5 shape: [T*B = 16000, 1280] x [1280, 2560]
        L = enc.layers[1][0]
        M = 16000
        xg = torch.from_numpy(synth.codes(8, (M, L.I))).to(dev)
        gx = torch.empty((M, 4 * L.H), dtype=torch.int32, device=dev)
        tg = timed(lambda: q.input_projection(L, xg, gx), 20, warm=3)
        gops = 2.0 * M * L.I * 4 * L.H
        extra["input_projection_gemm"] = {"M": M, "K": L.I, "N": 4 * L.H, "ms": tg * 1e3, "TOPs": gops / tg / 1e12,
                                          "frac_int8_mfma": gops / tg / 1e12 / INT8_MFMA_PEAK_TOPS}

    # ---------------------------------------------------------------- CPU oracle on a bounded slice
    if not args.no_cpu and args.leg in ("all",):
        import oracle
        from oracle import models as omodels
        Bc, Tc = min(oracle.get_max_threads(), 16), 12
        mo = synth.make_model(4)
        t0 = time.perf_counter()
        layers, proj = omodels.encoder_from_float(mo)
        M_o = omodels.model_from_float(mo)
        t_build = time.perf_counter() - t0
        fc = synth.features(4, Tc, Bc, mo.feat_dim)
        t0 = time.perf_counter()
        _, e_o = omodels.encoder_forward(layers, proj, fc, mo.alpha_x)
        oracle.decode(M_o, e_o, W, MAX_SYM)
        t_cpu = time.perf_counter() - t0
        result["cpu_baseline"] = {"value": t_cpu / (Bc * Tc * FRAME_SEC), "unit": "s/s", "cores": Bc,
                                  "kind": "oracle",
                                  "sample": f"same network, B={Bc} utterances x T={Tc} frames, beam {W}, max {MAX_SYM} labels/frame "
                                            f"({t_cpu:.1f} s of CPU work; weight quantization {t_build:.1f} s excluded)"}

    result["extra"] = extra
    if "value" not in result:
        result["value"] = None
        result["ms_per_step"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
