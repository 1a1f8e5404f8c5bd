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
  roofline      the dominant kernel (the fused LSTM step at 1024 hypotheses, the
                two grouped launches of one decoding round) against the dense int8
                MFMA peak, timed with HIP events on the launch stream;
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
    ap.add_argument("--no-graph", action="store_true",
                    help="time the kernel legs with direct launches instead of HIP-graph replays (for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (utterances are independent and would "
              "shard across GPUs without any collective). Run with --gpus 1.", file=sys.stderr)
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

    def timed_graph(fn, per_graph, replays=5):
        """Seconds per call of fn with the host out of the loop: per_graph launches are captured
        into one HIP graph (kernel launches only) and the replays are bracketed by HIP events on
        the launch stream."""
        if args.no_graph:
            return timed(fn, per_graph * replays, warm=3)
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(per_graph):
                fn()
        g.replay()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(replays):
            g.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / (replays * per_graph) * 1e-3

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
        enc.check()   # outside the timed region: no bounded wait of the persistent recurrence ran out
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
        # decoder time against the beam width (same encoder output, 200 frames): how search cost grows with W
        Ts = min(T, 200)
        es = e[:Ts].contiguous()
        sweep_w = []
        for Wb in (1, 2, 4, 8, 16):
            wsb = torch.empty(q.decode_workspace(G, Ts, B, Wb, MAX_SYM), dtype=torch.uint8, device=dev)
            tb = timed(lambda: q.decode(G, es, Wb, MAX_SYM, max_len=Ts * MAX_SYM, workspace=wsb), 1, warm=1)
            sweep_w.append({"beam": Wb, "decoder_ms_per_1000_frames": tb * 1e3 * 1000.0 / Ts,
                            "decoder_rtf": tb / (B * Ts * FRAME_SEC)})
            del wsb
        extra["beam_sweep"] = sweep_w
        # the early-stop variant of the search (same beams; rounds without a live hypothesis return at once)
        es_rows = []
        for Wb in (1, 16):
            wsb = torch.empty(q.decode_workspace(G, Ts, B, Wb, MAX_SYM), dtype=torch.uint8, device=dev)
            tf = timed(lambda: q.decode(G, es, Wb, MAX_SYM, max_len=Ts * MAX_SYM, workspace=wsb), 1, warm=1)
            te = timed(lambda: q.decode(G, es, Wb, MAX_SYM, max_len=Ts * MAX_SYM, workspace=wsb,
                                        flags=q.DECODE_EARLY_STOP), 1, warm=1)
            es_rows.append({"beam": Wb, "fixed_rounds_ms_per_1000_frames": tf * 1e3 * 1000.0 / Ts,
                            "early_stop_ms_per_1000_frames": te * 1e3 * 1000.0 / Ts})
            del wsb
        extra["early_stop"] = {"rows": es_rows,
                               "note": "a round dies only when no utterance of the batch picked a label in the round before: "
                                       "with beam 16 the 16 picks of a round always include labels, so nothing is skipped "
                                       "and the flag costs its loads; greedy search (beam 1) on this model skips most rounds"}
        # the paper's own search (Sec. 2): alignment-length synchronous with recombination, one joint + one network
        # advance per alignment step instead of up to five joints and four advances per frame
        alsd_rows = []
        for u_max in (T // 2, T):
            wsa = torch.empty(q.decode_alsd_workspace(G, T, B, W, u_max), dtype=torch.uint8, device=dev)
            ta = timed(lambda: q.decode_alsd(G, e, W, u_max, max_len=u_max, workspace=wsa), 1, warm=1)
            la = q.decode_alsd(G, e, W, u_max, max_len=u_max, workspace=wsa)[1].cpu().numpy()
            alsd_rows.append({"beam": W, "u_max": u_max, "iterations": T + u_max, "decoder_ms": ta * 1e3,
                              "decoder_rtf": ta / audio, "mean_labels_best_hyp": float(la[:, 0].mean())})
            del wsa
        extra["alsd"] = {"rows": alsd_rows,
                         "note": "same networks and encoder output as the headline; label cap u_max per utterance; the launch "
                                 "sequence has T + u_max iterations, those after the last live hypothesis return at once"}
        # Fig. 2(b) of the paper on this machine: decoder time of the paper's own search against the beam width
        # (200 frames, label cap T/2), with and without the reuse of cached hypotheses, and how often a label pick
        # found its sequence in the beam
        sweep_a = []
        for Wb in (1, 2, 4, 8, 16):
            um = Ts // 2
            wsa = torch.empty(q.decode_alsd_workspace(G, Ts, B, Wb, um), dtype=torch.uint8, device=dev)
            ta = timed(lambda: q.decode_alsd(G, es, Wb, um, max_len=um, workspace=wsa), 1, warm=1)
            st = torch.zeros(2, dtype=torch.int32, device=dev)
            tr = timed(lambda: q.decode_alsd(G, es, Wb, um, max_len=um, workspace=wsa, flags=q.ALSD_REUSE), 1, warm=1)
            q.decode_alsd(G, es, Wb, um, max_len=um, workspace=wsa, flags=q.ALSD_REUSE, stats=st)
            n_req, n_hit = (int(v) for v in st.cpu())
            sweep_a.append({"beam": Wb, "decoder_ms_per_1000_frames": ta * 1e3 * 1000.0 / Ts, "decoder_rtf": ta / (B * Ts * FRAME_SEC),
                            "with_reuse_ms_per_1000_frames": tr * 1e3 * 1000.0 / Ts, "label_picks": n_req, "reused": n_hit})
            del wsa
        extra["alsd_beam_sweep"] = {"rows": sweep_a,
                                    "note": "alignment-length synchronous search, label cap T/2; 'reused' = label picks whose sequence a live "
                                            "hypothesis of the beam already held (Sec. 4.1's reuse of cached hypotheses): they become copied "
                                            "rows of the advance; the advance is one dense launch per layer over all slots, so on this "
                                            "machine a reused row costs what an advanced one costs"}
        # worst case for the time-synchronous search: the blank's joint bias lowered until every pick of every round
        # is a label, so all four advances of a frame run over full lists (the headline model picks 15, 1, 15, 1 of 16)
        import copy
        m_lab = copy.deepcopy(m)
        m_lab.joint_out.bias = m_lab.joint_out.bias.copy()
        m_lab.joint_out.bias[0] -= 8.0
        G_lab = gmodel.model_from_float(m_lab, dev)
        wsl = torch.empty(q.decode_workspace(G_lab, Ts, B, W, MAX_SYM), dtype=torch.uint8, device=dev)
        tl = timed(lambda: q.decode(G_lab, es, W, MAX_SYM, max_len=Ts * MAX_SYM, workspace=wsl), 1, warm=1)
        ll = q.decode(G_lab, es, W, MAX_SYM, max_len=Ts * MAX_SYM, workspace=wsl)[1].cpu().numpy()
        extra["decode_all_labels"] = {"decoder_ms_per_1000_frames": tl * 1e3 * 1000.0 / Ts, "mean_labels_best_hyp_per_frame": float(ll[:, 0].mean()) / Ts,
                                      "note": "same networks with the blank made improbable: every round's 16 picks are labels "
                                              "(4 labels per frame), the upper bound of the decoder's time per frame"}
        del wsl, G_lab, m_lab
        del feats, ws_dec, e, es, out
        # the same pipeline with the layer shapes of the paper's Sec. 2 (340 features, prediction network and
        # source LM 1 x 768, external LM 2 x 2048 + bottleneck 256, fusion weights 0.7 / 0.5 / 0.2), all 4-bit
        m5 = synth.make_model(5)
        enc5 = gmodel.Encoder(m5, dev)
        G5 = gmodel.model_from_float(m5, dev)
        feats5 = torch.from_numpy(synth.features(5, T, B, m5.feat_dim)).to(dev)
        ws5 = torch.empty(q.decode_workspace(G5, T, B, W, MAX_SYM), dtype=torch.uint8, device=dev)
        _, e5 = enc5.forward(feats5)
        t_enc5 = timed(lambda: enc5.forward(feats5), 1, warm=0)
        t_dec5 = timed(lambda: q.decode(G5, e5, W, MAX_SYM, max_len=T * MAX_SYM, workspace=ws5), 1, warm=1)
        extra["paper_shapes"] = {"workload": f"Sec. 2 shapes, all 4-bit: 6x bi-LSTM-640 over 340 features, pred 1x768, source LM "
                                             f"1x768, external LM 2x2048 + bottleneck 256, beam {W}, max {MAX_SYM} labels/frame, "
                                             f"B={B} x T={T}",
                                 "encoder_ms": t_enc5 * 1e3, "decoder_ms": t_dec5 * 1e3,
                                 "rtf": (t_enc5 + t_dec5) / audio}
        del m5, enc5, G5, ws5, e5
        # ... and with the precision map of Sec. 3.2: 8-bit features, first encoder layer, encoder projection,
        # prediction-network output layer and joint output layer (8-bit weights straight onto the int8 MFMA)
        m6 = synth.make_model(5, mixed=True)
        enc6 = gmodel.Encoder(m6, dev)
        G6 = gmodel.model_from_float(m6, dev)
        ws6 = torch.empty(q.decode_workspace(G6, T, B, W, MAX_SYM), dtype=torch.uint8, device=dev)
        _, e6 = enc6.forward(feats5)
        t_enc6 = timed(lambda: enc6.forward(feats5), 1, warm=0)
        t_dec6 = timed(lambda: q.decode(G6, e6, W, MAX_SYM, max_len=T * MAX_SYM, workspace=ws6), 1, warm=1)
        extra["paper_shapes_mixed_precision"] = {"workload": "the same, first encoder layer and the RNN-T's linear layers at 8 bits (Sec. 3.2)",
                                                 "encoder_ms": t_enc6 * 1e3, "decoder_ms": t_dec6 * 1e3,
                                                 "rtf": (t_enc6 + t_dec6) / audio}
        del m6, enc6, G6, feats5, ws6, e6

    # ---------------------------------------------------------------- kernel legs
    if args.leg in ("all", "kernels"):
        def mk_state(n, H):
            return (torch.from_numpy(synth.codes(1, (n, H))).to(dev), torch.from_numpy(synth.normal(2, (n, H), 0.5)).to(dev))

        def clone_lstm(L):
            cm = lambda mq: q.QMat(mq.packed.clone(), mq.row_scale.clone(), mq.rows, mq.cols, mq.layout)
            return q.Lstm(cm(L.w_ih), cm(L.w_hh), L.bias.clone(), L.x_scale, L.h_scale, L.h_inv_scale)

        def round_groups(N, fresh_weights=False, mm=None, GG=None):
            """The two LSTM launches of one decoding round at N hypotheses, as qrnnt_decode issues them:
            first layers of the prediction network and of both LMs (input part looked up in the per-token
            table of input projections), then the second layers of both LMs.  fresh_weights: private
            copies of every weight tensor (for the cache-cold rotation)."""
            mm, GG = (m, G) if mm is None else (mm, GG)
            tok = torch.from_numpy(synth.token_ids(3, (N,), mm.V)).to(dev)
            parent = torch.from_numpy(synth.parent_perm(4, max(N // W, 1), min(W, N))).to(dev)
            groups = []
            for layer_idx in (0, 1):
                nets = [net for net in (GG.pred, GG.lm_src, GG.lm_ext) if len(net.layers) > layer_idx]
                steps, ops, byt = [], 0.0, 0.0
                for net in nets:
                    L = clone_lstm(net.layers[layer_idx]) if fresh_weights else net.layers[layer_idx]
                    hp, cp = mk_state(N, L.H)
                    d = dict(L=L, h_prev=hp, c_prev=cp, parent=parent, N=N,
                             h_next=torch.empty((N, L.H), dtype=torch.int8, device=dev),
                             c_next=torch.empty((N, L.H), dtype=torch.float32, device=dev))
                    if layer_idx == 0:
                        d["x_codes"], d["x_row"] = net.embed_codes, tok
                        d["gx"] = q.input_projection(L, net.embed_codes)[0]
                        d["gx_table"] = q.input_table(L, d["gx"])
                        k_in = 0
                        byt += mm.V * 4 * L.H * 4   # the table of per-token int32 sums
                    else:
                        d["x_codes"] = torch.from_numpy(synth.codes(5, (N, L.I))).to(dev)
                        k_in = L.I
                        byt += 4 * L.H * L.I / 2 + N * L.I
                    steps.append(d)
                    ops += 2.0 * 4 * L.H * (k_in + L.H) * N
                    # W_hh, scales and bias, hidden codes in/out, fp32 cell state in/out, parent indices
                    byt += 4 * L.H * L.H / 2 + 4 * L.H * 12 + N * L.H * (1 + 1 + 4 + 4) + 4 * N
                groups.append((q.StepGroup(steps), ops, byt))
            return groups

        # ---- decoding-round launches at 64 utterances x beam 16 = 1024 hypotheses (matrix-core bound)
        names = ("lstm_step_pipe_kernel<USE_GX=true,TAB=true>: pred L1 + 2 x LM L1, input part from the token table",
                 "lstm_step_pipe_kernel<USE_GX=false>: 2 x LM L2")
        launches, tot_ops, tot_t = [], 0.0, 0.0
        for name, (grp, ops, byt) in zip(names, round_groups(B * W)):
            t = timed_graph(grp.launch, 50)
            launches.append({"kernel": name, "avg_launch_us": t * 1e6, "ops": ops, "TOPs": ops / t / 1e12,
                             "frac_int8_mfma": ops / t / 1e12 / INT8_MFMA_PEAK_TOPS, "algorithmic_bytes": byt})
            tot_ops += ops
            tot_t += t
        ach = tot_ops / tot_t / 1e12
        result["roofline"] = {"bound": "mfma",
                              "kernel": "lstm_step_pipe_kernel (fused W4A4 LSTM step), the two launches of one decoding "
                                        f"round at N={B * W} hypotheses",
                              "achieved": ach, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                              "frac": ach / INT8_MFMA_PEAK_TOPS, "traffic": None,
                              "avg_launch_us": tot_t / 2 * 1e6, "ops_per_launch": tot_ops / 2, "launches": launches}
        tr = os.path.join(ROOT, "profiles", "lstm_step_pipe_kernel_decode_round_hbm_traffic.txt")
        if os.path.exists(tr):   # HBM bytes per launch from the committed rocprofv3 --pmc summary (counters cannot run here)
            import re
            hit = re.search(r"^hbm_bytes_per_launch:\s*(\d+)", open(tr).read(), re.M)
            result["roofline"]["traffic"] = int(hit.group(1)) if hit else None
            result["roofline"]["traffic_source"] = ("profiles/lstm_step_pipe_kernel_decode_round_hbm_traffic.txt: rocprofv3 --pmc "
                                                    "FETCH_SIZE / WRITE_SIZE of these two launches, calibrated on a copy; a committed "
                                                    "measurement of the same kernels, not taken in this run")

        # ---- what the matrix unit itself does: register-only rates of the instruction forms that can carry the
        # contraction exactly (codes in [-8, 7] are exact in int8 and fp8-E4M3, sums stay below 2^24)
        rates = q.diag_mfma_rates(20000, dev)
        best_i8 = max(t for n, t in rates if n.startswith("int8"))
        extra["mfma_forms"] = {"rows": [{"form": n, "TOPs": t, "frac_of_published_int8_peak": t / INT8_MFMA_PEAK_TOPS} for n, t in rates],
                               "int8_peak_at_measured_clock_TOPs": best_i8,
                               "implied_clock_GHz": best_i8 * 1e12 / (2048.0 * 4 * 256) / 1e9,
                               "note": "two workgroups per CU, 8 accumulator chains per wave (4 of the 32-row forms), two instructions per "
                                       "chain and loop iteration, no memory traffic, loop body checked to hold nothing but the matrix "
                                       "instructions. The best int8 rate gives the clock (2048 op/clk/SIMD). The fp6 forms hold the codes "
                                       "exactly (E2M3: -7.5..7.5 in steps of 0.5 above 4; E3M2: every integer up to 8), fp8-E4M3 too; "
                                       "fp4-E2M1 does not (no 5 and no 7). The 'chunk loop' rows run the same instructions in a loop "
                                       "shaped like the contraction kernels' 128-column chunk without its global loads (a barrier, the "
                                       "wave's operand reads from LDS for a 64 x 64 tile, the nibble unpack where the form needs one, "
                                       "three workgroups per CU): what the matrix unit and LDS allow together; the kernels' own "
                                       "rates are in roofline.launches"}
        result["roofline"]["peak_at_measured_clock"] = best_i8
        result["roofline"]["frac_of_peak_at_measured_clock"] = ach / best_i8

        # ---- beam-16 regime (one utterance, N = 16): weight streaming, against HBM
        byt16, t16 = 0.0, 0.0
        for grp, ops, byt in round_groups(16):
            t16 += timed_graph(grp.launch, 100)
            byt16 += byt
        extra["step_n16"] = {"kernel": "lstm_step_small_kernel, the two launches of one decoding round at N=16",
                             "us_per_round": t16 * 1e6, "algorithmic_bytes_per_round": byt16,
                             "GBps": byt16 / t16 / 1e9, "frac_hbm": byt16 / t16 / 1e9 / HBM_PEAK_GBPS,
                             "note": "weights re-read every round; warm (the 18 MB of weights stay in L2 / MALL)"}

        # ---- N = 16 with the layer shapes of Sec. 2 (external LM 2 x 2048: 25 MB of weights): three times the bytes
        # per launch for the same launch and latency overhead
        m5k = synth.make_model(5)
        G5k = gmodel.model_from_float(m5k, dev)
        byt5, t5 = 0.0, 0.0
        for grp, ops, byt in round_groups(16, mm=m5k, GG=G5k):
            t5 += timed_graph(grp.launch, 100)
            byt5 += byt
        extra["step_n16_paper_shapes"] = {"kernel": "the same two launches with the Sec. 2 shapes (pred 768, source LM 768, "
                                                    "external LM 2 x 2048)",
                                          "us_per_round": t5 * 1e6, "algorithmic_bytes_per_round": byt5,
                                          "GBps": byt5 / t5 / 1e9, "frac_hbm": byt5 / t5 / 1e9 / HBM_PEAK_GBPS}
        del m5k, G5k

        # ---- the same at N = 16 with the weights coming from HBM: 28 private copies of all weight tensors
        # (28 x 13.3 MB, more than the 256 MB MALL) visited in turn, so no launch finds its weights in a cache
        copies = [round_groups(16, fresh_weights=True) for _ in range(28)]

        def cold_round():
            for grps in copies:
                for grp, _, _ in grps:
                    grp.launch()

        tcold = timed_graph(cold_round, 2, replays=3) / len(copies)
        extra["step_n16_cold"] = {"us_per_round": tcold * 1e6, "GBps": byt16 / tcold / 1e9,
                                  "frac_hbm": byt16 / tcold / 1e9 / HBM_PEAK_GBPS,
                                  "note": "28 rotating weight copies (372 MB > MALL): every launch streams its weights from HBM"}
        del copies

        # ---- sweep of the hypothesis count: where weight streaming hands over to the matrix cores
        sweep = []
        for Ns in (16, 32, 64, 128, 256, 1024, 4096):
            ts, ops_s, byt_s = 0.0, 0.0, 0.0
            for grp, ops, byt in round_groups(Ns):
                ts += timed_graph(grp.launch, 50)
                ops_s += ops
                byt_s += byt
            sweep.append({"N": Ns, "us_per_round": ts * 1e6, "TOPs": ops_s / ts / 1e12, "GBps": byt_s / ts / 1e9})
        extra["step_round_sweep"] = sweep

        # ---- a plain device copy of known size: the HBM rate this machine sustains, and the kernel that
        # calibrates the FETCH_SIZE / WRITE_SIZE counters of the profiles
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        tc = timed(lambda: dst.copy_(src), 10, warm=2)
        extra["hbm_copy_reference"] = {"bytes_read": src.numel(), "bytes_written": src.numel(), "us": tc * 1e6,
                                       "GBps": 2 * src.numel() / tc / 1e9}
        del src, dst

        # ---- input-projection GEMM, encoder layers 2-6 shape: [T*B, 1280] x [1280, 2560] at configuration 1's
        # M = 16000 (32 utterances x 500 frames) and configuration 4's M = 64000 (64 x 1000: 656 MB of int32 sums,
        # more than the 256 MB cache in front of HBM holds)
        L = enc.layers[1][0]
        gemm_rows = []
        for M in (16000, 64000):
            xg = torch.from_numpy(synth.codes(8, (M, L.I))).to(dev)
            gx = torch.empty((M, 4 * L.H), dtype=torch.int32, device=dev)
            tg = timed_graph(lambda: q.input_projection(L, xg, gx), 20 if M <= 16000 else 6)
            gops = 2.0 * M * L.I * 4 * L.H
            gbytes = M * L.I + 4 * L.H * L.I / 2 + M * 4 * L.H * 4
            gemm_rows.append({"M": M, "K": L.I, "N": 4 * L.H, "us": tg * 1e6, "TOPs": gops / tg / 1e12,
                              "frac_int8_mfma": gops / tg / 1e12 / INT8_MFMA_PEAK_TOPS,
                              "algorithmic_bytes": gbytes, "GBps": gbytes / tg / 1e9})
            del xg, gx
        extra["input_projection_gemm"] = dict(gemm_rows[0], rows=gemm_rows)

        # ---- the encoder stack alone at the sizes of configuration 1: 32 utterances x 500 frames, and one utterance
        rows = []
        for (Be, Te) in ((32, 500), (1, 500)):
            fe = torch.from_numpy(synth.features(4, Te, Be, m.feat_dim)).to(dev)
            enc.workspace(Te, Be, dev)
            te = timed(lambda: enc.forward(fe), 3, warm=1)
            rows.append({"B": Be, "T": Te, "ms": te * 1e3, "rtf": te / (Be * Te * FRAME_SEC),
                         "us_per_layer_step": te * 1e6 / (len(enc.layers) * Te)})
            del fe
        extra["encoder_stack"] = {"rows": rows,
                                  "note": "6 bidirectional layers + projection; us_per_layer_step = time / (6 layers x T steps): both "
                                          "directions of a layer advance in the same persistent launch, input projections included"}

        # ---- what one step of the persistent recurrence costs when there is next to nothing to compute: a layer of
        # 32 cells (two workgroups per direction that wait for each other's hidden codes every step) over 2000 steps,
        # i.e. the exchange latency (publish -> visible -> polled) that every step of the encoder pays
        Lt = gmodel.lstm_from_float(synth._lstm(np.random.default_rng(5), 16, 32), gmodel.S_H, dev)
        Tf = 2000
        xf = torch.from_numpy(synth.codes(9, (Tf, 16, 16))).to(dev)
        wsf = torch.empty(q.lstm_layer_workspace(Lt, Tf, 16), dtype=torch.uint8, device=dev)
        hof = torch.empty((Tf, 16, 32), dtype=torch.int8, device=dev)
        tf_ = timed(lambda: q.lstm_layer(Lt, xf, h_out=hof, workspace=wsf), 3, warm=1)
        assert q.layer_error_flag(wsf, wsf.numel()) == 0
        extra["recurrence_exchange_floor"] = {"us_per_step": tf_ * 1e6 / Tf,
                                              "note": "H = 32 (2 workgroups exchanging tagged words), B = 16, T = 2000, input projection included "
                                                      "(0.1 % of the time): the latency floor of a recurrence step; compare "
                                                      "encoder_stack.us_per_layer_step"}
        del xf, wsf, hof

    # ---------------------------------------------------------------- CPU oracle on a bounded slice
    if not args.no_cpu and args.leg in ("all",):
        import oracle
        from oracle import models as omodels
        Bc, Tc = min(oracle.get_max_threads(), 16), 40
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

        # one thread on one utterance, for the per-core rate
        oracle.set_threads(1)
        f1 = synth.features(4, 10, 1, mo.feat_dim)
        t0 = time.perf_counter()
        _, e_1 = omodels.encoder_forward(layers, proj, f1, mo.alpha_x)
        oracle.decode(M_o, e_1, W, MAX_SYM)
        t_1 = time.perf_counter() - t0
        oracle.set_threads(Bc)
        extra["cpu_oracle_single_thread"] = {"value": t_1 / (10 * FRAME_SEC), "unit": "s/s", "cores": 1,
                                             "sample": f"B=1 x T=10 frames ({t_1:.1f} s)"}

        # Sec. 4.1's reuse of cached hypotheses, counted by the oracle on a slice: network advances a search without
        # a cache makes, with the current beam as the cache (what the GPU's QRNNT_ALSD_REUSE does), and with every
        # sequence ever extended kept
        e_c = np.ascontiguousarray(e_o[:20, :4])
        rows_c = []
        for Wc in (1, 4, 16):
            r1 = oracle.decode_alsd_cached(M_o, e_c, Wc, 10, 1)
            r2 = oracle.decode_alsd_cached(M_o, e_c, Wc, 10, 2)
            rows_c.append({"beam": Wc, "advances_without_cache": int(r1[3].sum()), "with_beam_as_cache": int(r1[4].sum()),
                           "with_unbounded_cache": int(r2[4].sum())})
        extra["hypothesis_cache_oracle"] = {"rows": rows_c, "sample": "ALSD, 4 utterances x 20 frames, label cap 10, config-4 networks"}

    result["extra"] = extra
    if "value" not in result:
        result["value"] = None
        result["ms_per_step"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
