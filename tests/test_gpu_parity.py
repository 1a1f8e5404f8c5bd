"""Parity of the HIP path with the CPU oracle, call by call through the C ABI.

Every kernel is fed the same seeded inputs as the oracle (teacher forcing: a
rounding tie in one step cannot leak into the next comparison).  Bars:
int32 accumulators, packed bytes, codes of weights/inputs and beam selections
are bit-exact; fp32 gates and cell states within 1e-5 relative (+1e-6 absolute
at zero crossings); requantised hidden codes agree on >= 99.99 % of entries and
differ by one code only where the real value sits on a rounding tie; log-probs
and fused scores within 1e-3 absolute (observed ~1e-6).
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import models
from paper_2206_07882_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
S_H = float(np.float32(1) / np.float32(7))


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.detach().cpu().numpy()


def assert_codes_close(got, ref, real, what, min_agree=0.9999):
    """Codes equal except at rounding ties of `real` (= value * inv_step, fp64)."""
    got = got.astype(np.int32); ref = ref.astype(np.int32)
    if got.size == 0:
        return
    bad = got != ref
    frac = 1.0 - bad.mean()
    assert frac >= min_agree, f"{what}: only {frac:.6f} of codes agree"
    if bad.any():
        assert np.abs(got - ref)[bad].max() == 1, f"{what}: code differs by more than 1"
        dist = np.abs(real[bad] - np.floor(real[bad]) - 0.5)
        assert dist.max() < 1e-4, f"{what}: mismatch away from a rounding tie ({dist.max()})"


def assert_rel(got, ref, what, rtol=1e-5, atol=1e-6):
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    lim = rtol * np.abs(ref.astype(np.float64)) + atol
    assert np.all(err <= lim), f"{what}: max excess {np.max(err - lim):.3e}"


# ------------------------------------------------------------------ pack / quantize

@pytest.mark.parametrize("rows,cols", [(64, 32), (256, 64), (2560, 240), (48, 256), (46, 256), (16, 32), (4, 16)])
def test_pack_roundtrip_and_canonical_bytes(gpu_lib, rows, cols):
    q = gpu_lib
    codes = synth.codes(11 + rows + cols, (rows, cols), -8, 7)
    for layout in (q.LAYOUT_ROWMAJOR, q.LAYOUT_TILED) + ((q.LAYOUT_TILED_GATES,) if rows % 4 == 0 else ()):
        m = q.pack_int4(dev(codes), layout)
        assert np.array_equal(host(q.unpack_int4(m)), codes), f"layout {layout}"
        if layout == q.LAYOUT_ROWMAJOR:
            cp = (cols + 63) // 64 * 64
            assert np.array_equal(host(m.packed).reshape(rows, cp // 2), oracle.pack_rows(codes, cp))


def _tiled_blob(codes, gates):
    """The TILED / TILED_GATES blob written out from the layout notes of the header, in numpy."""
    rows, cols = codes.shape
    H = rows // 4
    rp = (rows + 63) // 64 * 64 if gates else (rows + 15) // 16 * 16
    nkc = (cols + 127) // 128
    padded = np.zeros((rp, nkc * 128), np.int8)
    if gates:
        for j in range(H):
            q, a, b = j // 16, (j % 16) // 4, j % 4
            for g in range(4):
                padded[64 * q + 16 * b + 4 * a + g, :cols] = codes[g * H + j]
    else:
        padded[:rows, :cols] = codes
    blob = np.zeros((rp // 16, nkc, 64, 16), np.uint8)
    nib = (padded.astype(np.int16) & 0xF).astype(np.uint8)
    for lane in range(64):
        r, kq = lane % 16, lane // 16
        lo = nib[r::16, :].reshape(rp // 16, nkc, 128)[:, :, 16 * kq:16 * kq + 16]
        hi = nib[r::16, :].reshape(rp // 16, nkc, 128)[:, :, 64 + 16 * kq:64 + 16 * kq + 16]
        blob[:, :, lane, :] = lo | (hi << 4)
    return blob.reshape(-1)


@pytest.mark.parametrize("rows,cols", [(64, 32), (2560, 240), (48, 256), (46, 256), (4, 16), (3072, 768)])
def test_pack_tiled_bytes_follow_the_documented_layout(gpu_lib, rows, cols):
    q = gpu_lib
    codes = synth.codes(15 + rows + cols, (rows, cols), -8, 7)
    m = q.pack_int4(dev(codes), q.LAYOUT_TILED)
    assert np.array_equal(host(m.packed), _tiled_blob(codes, False))
    if rows % 4 == 0:
        m = q.pack_int4(dev(codes), q.LAYOUT_TILED_GATES)
        assert np.array_equal(host(m.packed), _tiled_blob(codes, True))


@pytest.mark.parametrize("rows,cols", [(64, 32), (3072, 768), (46, 256)])
def test_pack_from_fp32_matches_oracle_quantizer(gpu_lib, rows, cols):
    q = gpu_lib
    w = synth.normal(21 + rows, (rows, cols), 1.0 / np.sqrt(cols))
    w[1, :] = 0.0                      # an all-zero row
    w[2, 3] = np.abs(w[2]).max() * 0.5  # an exact tie at 3.5 steps
    ref_codes, ref_scale = oracle.quantize_weight_rows(w)
    for layout in (q.LAYOUT_TILED, q.LAYOUT_ROWMAJOR) + ((q.LAYOUT_TILED_GATES,) if rows % 4 == 0 else ()):
        m = q.pack_int4(dev(w), layout)
        assert np.array_equal(host(q.unpack_int4(m)), ref_codes)
        assert np.array_equal(host(m.row_scale), ref_scale)


def test_quantize_act_bit_exact_including_ties(gpu_lib):
    q = gpu_lib
    x = synth.normal(31, (500 * 3 * 240 + 3,), 1.0)
    x[:9] = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 100.0, -100.0, 0.0, 6.5], np.float32) * np.float32(4.0 / 7.0)
    inv = float(np.float32(7) / np.float32(4))
    n = x.size - 3
    # aligned body and a ragged tail
    assert np.array_equal(host(q.quantize_act(dev(x[:n]), inv)), oracle.quant_sym4(x[:n], inv))
    assert np.array_equal(host(q.quantize_act(dev(x[:n - 1]), inv)), oracle.quant_sym4(x[:n - 1], inv))
    assert np.array_equal(host(q.quantize_act(dev(x[:5]), 1.0)), oracle.quant_sym4(x[:5], 1.0))


# ------------------------------------------------------------------ linear

@pytest.mark.parametrize("rows,cols,N,lsm", [(256, 1280, 300, False), (256, 768, 16, False), (32, 64, 5, False),
                                             (46, 1024, 1024, True), (46, 1024, 16, True), (16, 64, 4, True),
                                             (46, 256, 37, False)])
def test_linear_parity(gpu_lib, rows, cols, N, lsm):
    q = gpu_lib
    w = synth.normal(41 + rows, (rows, cols), 1.0 / np.sqrt(cols))
    b = synth.normal(42 + rows, (rows,), 0.1)
    a = synth.codes(43 + N, (N, cols), -8, 7)
    P = oracle.Linear.from_float(w, b, S_H)
    m = q.pack_int4(dev(w), q.LAYOUT_TILED)
    y, acc = q.linear(m, dev(b), S_H, dev(a), log_softmax=lsm, want_acc=True)
    ry, racc = oracle.linear(P, a, want_acc=True)
    assert np.array_equal(host(acc), racc)
    if lsm:
        assert np.abs(host(y) - oracle.log_softmax(ry)).max() < 2e-5
    else:
        assert_rel(host(y), ry, "linear y")


@pytest.mark.parametrize("rows,cols,N", [(256, 2048, 40), (16, 64, 3), (48, 128, 17), (30, 96, 33)])
def test_linear_quant_parity(gpu_lib, rows, cols, N):
    """Linear layer fused with the quantizer of the layer it feeds (the bottleneck of the external LM,
    Sec. 2): codes must equal the oracle's quantizer applied to the oracle's linear output, except
    where the fp32 result sits on a rounding tie (then one code apart)."""
    q = gpu_lib
    w = synth.normal(61 + rows, (rows, cols), 1.0 / np.sqrt(cols))
    b = synth.normal(62 + rows, (rows,), 0.1)
    a = synth.codes(63 + N, (N, cols), -8, 7)
    P = oracle.Linear.from_float(w, b, S_H)
    m = q.pack_int4(dev(w), q.LAYOUT_TILED)
    inv = float(np.float32(7.0) / np.float32(0.6))     # boundary inside the output range: the clamp is exercised
    got = host(q.linear_quant(m, dev(b), S_H, dev(a), inv))
    ry = oracle.linear(P, a)
    ref = oracle.quant_sym4(ry, inv)
    assert got.min() == -8 and got.max() == 7
    diff = got.astype(np.int32) - ref
    bad = np.nonzero(diff)
    assert len(bad[0]) <= max(1, got.size // 10000)
    t = ry[bad].astype(np.float64) * inv
    assert np.all(np.abs(diff[bad]) == 1) and np.all(np.abs(np.abs(t - np.floor(t)) - 0.5) < 1e-3)


# ------------------------------------------------------------------ LSTM step

_PAIRS = {}


def _lstm_pair(q, seed, I, H, s_x, std=None):
    """(oracle layer, GPU layer) from the same seeded float weights; built once per distinct argument set."""
    key = (seed, I, H, float(s_x), std)
    if key not in _PAIRS:
        _PAIRS[key] = _make_lstm_pair(q, seed, I, H, s_x, std)
    return _PAIRS[key]


def _make_lstm_pair(q, seed, I, H, s_x, std=None):
    sd_i = std if std is not None else 1.0 / np.sqrt(I)
    sd_h = std if std is not None else 1.0 / np.sqrt(H)
    w_ih = synth.normal(seed, (4 * H, I), sd_i)
    w_hh = synth.normal(seed + 1, (4 * H, H), sd_h)
    bias = synth.normal(seed + 2, (4 * H,), 0.1)
    L = oracle.Lstm.from_float(w_ih, w_hh, bias, s_x, S_H, 7.0)
    G = q.Lstm(q.pack_int4(dev(w_ih), q.LAYOUT_TILED_GATES), q.pack_int4(dev(w_hh), q.LAYOUT_TILED_GATES), dev(bias),
               float(np.float32(s_x)), S_H, 7.0)
    return L, G


def _check_step(dbg_g, hn_g, cn_g, ref, what):
    hn_r, cn_r, dbg_r = ref
    assert np.array_equal(host(dbg_g["accx"]), dbg_r["accx"]), what + " accx"
    assert np.array_equal(host(dbg_g["acch"]), dbg_r["acch"]), what + " acch"
    assert_rel(host(dbg_g["gates"]), dbg_r["gates"], what + " gates")
    assert_rel(host(cn_g), cn_r, what + " c")
    assert_codes_close(host(hn_g), hn_r, dbg_r["h_real"] * 7.0, what + " h codes")


@pytest.mark.parametrize("I,H,N", [(64, 64, 4), (32, 64, 2), (768, 768, 16), (256, 1024, 16), (1024, 1024, 37),
                                   (240, 640, 32), (1280, 640, 1)])
def test_lstm_step_parity_plain(gpu_lib, I, H, N):
    q = gpu_lib
    s_x = float(np.float32(1.25) / np.float32(7))
    L, G = _lstm_pair(q, 51 + I + H, I, H, s_x)
    x = synth.codes(52 + N, (N, I), -8, 7)
    hp = synth.codes(53 + N, (N, H), -7, 7)
    cp = synth.normal(54 + N, (N, H), 0.7)
    hn, cn, dbg = q.lstm_step(G, dev(x), dev(hp), dev(cp), debug=True)
    _check_step(dbg, hn, cn, oracle.lstm_step(L, x, hp, cp, debug=True), f"step {I}x{H}x{N}")


def test_lstm_step_parity_beam_shape_with_gather_and_mask(gpu_lib):
    """Prediction-network shape at 64 utterances x beam 16: embedding rows picked
    by token id, previous state picked by parent slot, blank-extended rows masked."""
    q = gpu_lib
    I = H = 768
    B, W, V = 64, 16, 46
    N = B * W
    s_x = float(np.float32(1.25) / np.float32(7))
    L, G = _lstm_pair(q, 61, I, H, s_x)
    emb = synth.codes(62, (V, I), -7, 7)
    tok = synth.token_ids(63, (N,), V)
    parent = synth.parent_perm(64, B, W)
    active = (np.random.default_rng(65).random(N) < 0.6).astype(np.uint8)
    hp = synth.codes(66, (N, H), -7, 7)
    cp = synth.normal(67, (N, H), 0.7)
    hn, cn, dbg = q.lstm_step(G, dev(emb), dev(hp), dev(cp), x_row=dev(tok), parent=dev(parent), active=dev(active),
                              debug=True)
    hn, cn = host(hn), host(cn)
    # the oracle checks a sample of rows one by one (rows are independent given their parent)
    rows = np.random.default_rng(68).choice(N, 96, replace=False)
    ref = oracle.lstm_step(L, emb[tok[rows]], hp[parent[rows]], cp[parent[rows]], active=active[rows], debug=True)
    act = active[rows].astype(bool)
    assert np.array_equal(host(dbg["accx"])[rows][act], ref[2]["accx"][act])
    assert np.array_equal(host(dbg["acch"])[rows][act], ref[2]["acch"][act])
    assert_rel(host(dbg["gates"])[rows][act], ref[2]["gates"][act], "gates")
    assert_rel(cn[rows], ref[1], "c")
    assert_codes_close(hn[rows][act], ref[0][act], (ref[2]["h_real"] * 7.0)[act], "h codes")
    # masked rows are exact copies of the parent slot, over the whole batch
    ina = active == 0
    assert np.array_equal(hn[ina], hp[parent[ina]]) and np.array_equal(cn[ina], cp[parent[ina]])


def _tiled_gate_col(H):
    """Column of gx that holds (cell j, gate g): the TILED_GATES row order of the header."""
    j = np.arange(H)
    base = 64 * (j // 16) + 16 * (j % 4) + 4 * ((j % 16) // 4)
    return base[None, :] + np.arange(4)[:, None]          # [gate, cell]


@pytest.mark.parametrize("I,H,M", [(240, 640, 77), (1280, 640, 300), (768, 768, 46), (64, 16, 5)])
def test_input_projection_exact(gpu_lib, I, H, M):
    q = gpu_lib
    L, G = _lstm_pair(q, 71 + I, I, H, 0.1)
    x = synth.codes(72 + M, (M, I), -8, 7)
    gx, acc = q.input_projection(G, dev(x), debug=True)
    ref = oracle.lstm_step(L, x, np.zeros((M, H), np.int8), np.zeros((M, H), np.float32), debug=True)[2]["accx"]
    assert np.array_equal(host(acc), ref)
    col = _tiled_gate_col(H)
    gxh = host(gx)
    for g in range(4):
        assert np.array_equal(gxh[:, col[g]], ref[:, g * H:(g + 1) * H]), f"gate {g}"


@pytest.mark.parametrize("N,use_gx", [(16, False), (16, True), (48, True), (144, False), (144, True), (256, True),
                                       (256, False), (16, "table"), (144, "table"), (256, "table"),
                                       (11, False), (11, "table"), (5, True)])
def test_lstm_step_group_parity(gpu_lib, N, use_gx):
    """Three independent steps in one launch (widths of the first layers of the
    prediction network and of two LMs, scaled down), inputs picked by token id from
    an embedding table; with use_gx the input part comes from the per-token table of
    input projections.  Both must reproduce the oracle's step on the looked-up rows."""
    q = gpu_lib
    V = 46
    shapes = [(128, 128), (64, 256), (64, 256)]
    s_x = float(np.float32(1.25) / np.float32(7))
    W = min(16, N)
    parent = synth.parent_perm(80 + N, N // W, W)
    tok = synth.token_ids(81 + N, (N,), V)
    active = (np.random.default_rng(82 + N).random(N) < 0.7).astype(np.uint8)
    steps, refs = [], []
    for i, (I, H) in enumerate(shapes):
        L, G = _lstm_pair(q, 90 + 10 * i, I, H, s_x)
        emb = synth.codes(91 + i, (V, I), -7, 7)
        hp = synth.codes(92 + i, (N, H), -7, 7)
        cp = synth.normal(93 + i, (N, H), 0.7)
        d = dict(L=G, x_codes=dev(emb), x_row=dev(tok), parent=dev(parent), active=dev(active), h_prev=dev(hp),
                 c_prev=dev(cp), N=N, h_next=torch.empty((N, H), dtype=torch.int8, device=DEV),
                 c_next=torch.empty((N, H), dtype=torch.float32, device=DEV))
        if use_gx:
            d["gx"] = q.input_projection(G, dev(emb))[0]
        if use_gx == "table":   # the fp32 form with scales and bias folded in
            d["gx_table"] = q.input_table(G, d["gx"])
        steps.append(d)
        refs.append(oracle.lstm_step(L, emb[tok], hp[parent], cp[parent], active=active, debug=True))
    q.StepGroup(steps).launch()
    for d, (hn_r, cn_r, dbg_r) in zip(steps, refs):
        assert_rel(host(d["c_next"]), cn_r, "c")
        act = active.astype(bool)
        assert_codes_close(host(d["h_next"])[act], hn_r[act], (dbg_r["h_real"] * 7.0)[act], "h codes")
        assert np.array_equal(host(d["h_next"])[~act], hn_r[~act])


def test_lstm_step_group_full_size_all_rows(gpu_lib):
    """The two grouped launches of one decoding round exactly as the benchmark times them (64 utterances x
    beam 16 = 1024 hypotheses; prediction network 768 and both LMs' first layers 1024 fed from the per-token
    table, then both LMs' second layers 1024 <- 1024), every hypothesis and every cell against the oracle.
    Each launch runs twice: as the benchmark runs it (the production build of the kernel variant) and with the
    debug outputs (the debug build of the same variant), whose int32 sums must be the oracle's bit for bit and
    whose states must be the production build's bit for bit."""
    q = gpu_lib
    V, W, B = 46, 16, 64
    N = B * W
    s_x = float(np.float32(1.25) / np.float32(7))
    parent = synth.parent_perm(180, B, W)
    tok = synth.token_ids(181, (N,), V)
    active = (np.random.default_rng(182).random(N) < 0.9).astype(np.uint8)
    act = active.astype(bool)
    for shapes, table in (([(768, 768), (256, 1024), (256, 1024)], True), ([(1024, 1024), (1024, 1024)], False)):
        steps, refs = [], []
        for i, (I, H) in enumerate(shapes):
            L, G = _lstm_pair(q, 190 + 10 * i + I, I, H, s_x if table else S_H)
            hp = synth.codes(192 + i, (N, H), -7, 7)
            cp = synth.normal(193 + i, (N, H), 0.7)
            d = dict(L=G, parent=dev(parent), active=dev(active), h_prev=dev(hp), c_prev=dev(cp), N=N,
                     h_next=torch.empty((N, H), dtype=torch.int8, device=DEV),
                     c_next=torch.empty((N, H), dtype=torch.float32, device=DEV))
            if table:
                emb = synth.codes(191 + i, (V, I), -7, 7)
                gx = q.input_projection(G, dev(emb))[0]
                d.update(x_codes=dev(emb), x_row=dev(tok), gx=gx, gx_table=q.input_table(G, gx))
                x_rows = emb[tok]
                # the table's integer form: the oracle's input sums of every token, bit for bit
                ref_tab = oracle.matmul_i32(L.w_ih, emb)
                col = _tiled_gate_col(H)
                for g4 in range(4):
                    assert np.array_equal(host(gx)[:, col[g4]], ref_tab[:, g4 * H:(g4 + 1) * H])
            else:
                x = synth.codes(194 + i, (N, I), -7, 7)
                d.update(x_codes=dev(x))
                x_rows = x
            steps.append(d)
            refs.append(oracle.lstm_step(L, x_rows, hp[parent], cp[parent], active=active, debug=True))
        q.StepGroup(steps).launch()
        prod = [(host(d["h_next"]).copy(), host(d["c_next"]).copy()) for d in steps]
        for d, (hn_r, cn_r, dbg_r) in zip(steps, refs):
            assert_rel(host(d["c_next"]), cn_r, "c")
            assert_codes_close(host(d["h_next"])[act], hn_r[act], (dbg_r["h_real"] * 7.0)[act], "h codes")
            assert np.array_equal(host(d["h_next"])[~act], hn_r[~act])
        # the debug build of the same variant
        for d in steps:
            H = d["L"].H
            d["h_next"] = torch.empty_like(d["h_next"]); d["c_next"] = torch.empty_like(d["c_next"])
            d["dbg_acch"] = torch.zeros((N, 4 * H), dtype=torch.int32, device=DEV)
            d["dbg_gates"] = torch.zeros((N, 4 * H), dtype=torch.float32, device=DEV)
            if not table:
                d["dbg_accx"] = torch.zeros((N, 4 * H), dtype=torch.int32, device=DEV)
        q.StepGroup(steps).launch()
        for d, (hn_r, cn_r, dbg_r), (hn_p, cn_p) in zip(steps, refs, prod):
            assert np.array_equal(host(d["dbg_acch"])[act], dbg_r["acch"][act]), "acch"
            if not table:
                assert np.array_equal(host(d["dbg_accx"])[act], dbg_r["accx"][act]), "accx"
            assert_rel(host(d["dbg_gates"])[act], dbg_r["gates"][act], "gates")
            assert np.array_equal(host(d["h_next"]), hn_p) and np.array_equal(host(d["c_next"]), cn_p)


@pytest.mark.parametrize("N,n_list", [(1024, 0), (1024, 1), (1024, 33), (1024, 64), (1024, 65), (1024, 100), (1024, 128),
                                      (1024, 129), (1024, 250), (1024, 300), (1024, 512), (1024, 700), (1024, 960),
                                      (1024, 1024), (512, 64), (256, 40), (144, 70), (128, 64), (128, 20), (48, 17),
                                      (32, 10), (16, 16), (16, 5)])
def test_lstm_step_group_listed(gpu_lib, N, n_list):
    """qrnnt_lstm_step_group_listed at the shapes of a decoding round (first layers from the per-token table, then
    the LMs' second layers): the listed hypotheses, in a seeded random order, must get the oracle's step (all of
    them, every cell), every other row of the outputs must keep what it held; once as the decoder launches it and
    once with the int32 sums of the recurrent part as a debug output, which must be the oracle's bit for bit.
    The list lengths walk through the kernel's ways of splitting a list over workgroups (32, 64 or 128 entries each) and their ragged ends; entries beyond the count
    hold out-of-range values, which must be harmless."""
    q = gpu_lib
    V, W = 46, 16
    s_x = float(np.float32(1.25) / np.float32(7))
    rng = np.random.default_rng(7000 + 7 * N + n_list)
    parent = synth.parent_perm(280 + N, N // W, W)
    tok = synth.token_ids(281 + N, (N,), V)
    active = (rng.random(N) < 0.9).astype(np.uint8)
    listed = rng.permutation(N)[:n_list].astype(np.int32)
    lst = np.empty((N, 4), np.int32)
    lst[:, 0] = rng.choice([-5, N, N + 1000, 2 ** 30], N)      # what follows the end of the list: out of range
    lst[:, 1] = rng.choice([-1, N, 2 ** 30], N)
    lst[:, 2] = rng.choice([-7, V, 2 ** 29], N)
    lst[:, 3] = 0
    lst[:n_list, 0] = listed
    lst[:n_list, 1] = parent[listed]
    lst[:n_list, 2] = tok[listed]
    cnt = dev(np.array([n_list], np.int32))
    rows = listed                                    # every listed hypothesis is checked
    act = active[rows].astype(bool)
    unlisted = np.setdiff1d(np.arange(N), listed)
    for shapes, table, with_dbg in (([(768, 768), (256, 1024), (256, 1024)], True, False),
                                    ([(1024, 1024), (1024, 1024)], False, False),
                                    ([(768, 768), (256, 1024), (256, 1024)], True, True),
                                    ([(1024, 1024), (1024, 1024)], False, True)):
        steps, refs = [], []
        for i, (I, H) in enumerate(shapes):
            L, G = _lstm_pair(q, 290 + 10 * i + I, I, H, s_x if table else S_H)
            hp = synth.codes(292 + i, (N, H), -7, 7)
            cp = synth.normal(293 + i, (N, H), 0.7)
            d = dict(L=G, parent=dev(parent), active=dev(active), h_prev=dev(hp), c_prev=dev(cp), N=N,
                     h_next=torch.full((N, H), 5, dtype=torch.int8, device=DEV),
                     c_next=torch.full((N, H), 123.0, dtype=torch.float32, device=DEV))
            if with_dbg:   # the debug build of the variant (and of its half- and quarter-width instances)
                d["dbg_acch"] = torch.full((N, 4 * H), -77, dtype=torch.int32, device=DEV)
            if table:
                emb = synth.codes(291 + i, (V, I), -7, 7)
                gx = q.input_projection(G, dev(emb))[0]
                d.update(x_codes=dev(emb), x_row=dev(tok), gx=gx, gx_table=q.input_table(G, gx))
                x_rows = emb[tok[rows]]
                l_dev = dev(lst)
            else:                      # no x_row: the entry's third word must not be used
                x = synth.codes(294 + i, (N, I), -7, 7)
                d.update(x_codes=dev(x))
                x_rows = x[rows]
                l_dev = dev(lst)
            steps.append(d)
            refs.append(oracle.lstm_step(L, x_rows, hp[parent[rows]], cp[parent[rows]], active=active[rows], debug=True)
                        if n_list else None)
        q.StepGroup(steps).launch(list=l_dev, n_list=cnt)
        for d, ref in zip(steps, refs):
            hn, cn = host(d["h_next"]), host(d["c_next"])
            assert np.all(hn[unlisted] == 5) and np.all(cn[unlisted] == 123.0), "a row outside the list was written"
            if ref is None:
                continue
            hn_r, cn_r, dbg_r = ref
            assert_rel(cn[rows], cn_r, "c")
            assert_codes_close(hn[rows][act], hn_r[act], (dbg_r["h_real"] * 7.0)[act], "h codes")
            assert np.array_equal(hn[rows][~act], hn_r[~act])
            if with_dbg:               # int32 sums of the listed rows bit for bit, nothing written for the others
                acc = host(d["dbg_acch"])
                assert np.array_equal(acc[rows][act], dbg_r["acch"][act]) and np.all(acc[unlisted] == -77)


def test_lstm_step_extreme_codes_no_overflow(gpu_lib):
    """All weights at code 7/-7 against all activations at -8: the largest |sum|."""
    q = gpu_lib
    I, H, N = 2048, 64, 16
    w_ih = np.full((4 * H, I), -8, np.int8); w_ih[::2] = 7
    w_hh = np.full((4 * H, H), -8, np.int8)
    ones = np.ones(4 * H, np.float32) * np.float32(1e-3)
    bias = np.zeros(4 * H, np.float32)
    L = oracle.Lstm(w_ih, ones, w_hh, ones, bias, 0.01, S_H, 7.0)
    G = q.Lstm(q.pack_int4(dev(w_ih), q.LAYOUT_TILED_GATES, dev(ones)),
               q.pack_int4(dev(w_hh), q.LAYOUT_TILED_GATES, dev(ones)), dev(bias), 0.01, S_H, 7.0)
    x = np.full((N, I), -8, np.int8)
    hp = np.full((N, H), -8, np.int8)
    cp = np.zeros((N, H), np.float32)
    hn, cn, dbg = q.lstm_step(G, dev(x), dev(hp), dev(cp), debug=True)
    ref = oracle.lstm_step(L, x, hp, cp, debug=True)
    assert np.array_equal(host(dbg["accx"]), ref[2]["accx"]) and host(dbg["accx"]).max() == 64 * I
    assert host(dbg["accx"]).min() == -56 * I
    assert np.array_equal(host(dbg["acch"]), ref[2]["acch"])


# ------------------------------------------------------------------ LSTM layer

@pytest.mark.parametrize("T,B,I,H,reverse", [(20, 2, 32, 64, False), (7, 3, 32, 64, True), (12, 32, 240, 640, False),
                                             (9, 32, 1280, 640, True), (16, 1, 240, 640, False)])
def test_lstm_layer_parity(gpu_lib, T, B, I, H, reverse):
    """Whole-utterance layer: input-projection GEMM bit-exact; then every time step
    is checked against one oracle step fed the GPU's own previous state, so a tie
    flip cannot cascade; the free-running oracle layer is compared as well."""
    q = gpu_lib
    s_x = float(np.float32(4) / np.float32(7)) if I in (32, 240) else S_H
    L, G = _lstm_pair(q, 71 + I + H, I, H, s_x)
    x = synth.codes(72 + T, (T, B, I), -8, 7)
    ld, off = 2 * H + 16, 16
    h_out = torch.full((T, B, ld), 55, dtype=torch.int8, device=DEV)
    need = q.lstm_layer_workspace(G, T, B)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = q.lstm_layer(G, dev(x), reverse=reverse, h_out=h_out, col_off=off, want_last=True, debug=True, workspace=ws)
    assert q.layer_error_flag(ws, need) == 0
    hg = host(out["h_out"]); cg = host(out["c_all"])
    assert np.all(hg[:, :, :off] == 55) and np.all(hg[:, :, off + H:] == 55)
    hg = hg[:, :, off:off + H]
    assert np.array_equal(host(out["accx"]).reshape(T * B, 4 * H), oracle.matmul_i32(L.w_ih, x.reshape(T * B, I)))
    order = range(T - 1, -1, -1) if reverse else range(T)
    hp = np.zeros((B, H), np.int8); cp = np.zeros((B, H), np.float32)
    for t in order:
        hr, cr, dbg = oracle.lstm_step(L, x[t], hp, cp, debug=True)
        assert_rel(cg[t], cr, f"c t={t}")
        assert_codes_close(hg[t], hr, dbg["h_real"] * 7.0, f"h t={t}")
        hp, cp = hg[t], cg[t]
    assert np.array_equal(host(out["h_last"]), hp) and np.array_equal(host(out["c_last"]), cp)
    free, _, _, _ = oracle.lstm_layer(L, x, reverse=reverse)
    agree = (free == hg).mean()
    assert agree >= (1.0 if T * B * H < 5000 else 0.999), f"free-running agreement {agree}"


@pytest.mark.parametrize("T,B,I,H", [(20, 2, 32, 64), (12, 32, 240, 640), (10, 64, 1280, 640), (6, 100, 240, 640),
                                     (25, 1, 240, 640), (5, 3, 64, 1024)])
def test_bilstm_layer_parity(gpu_lib, T, B, I, H):
    """Both directions in one launch (persistent recurrence, hidden codes exchanged
    between workgroups): input-projection + every step checked against one oracle
    step fed the GPU's own previous codes and the oracle's cell state of that chain."""
    q = gpu_lib
    s_x = float(np.float32(4) / np.float32(7)) if I in (32, 240) else S_H
    Lf, Gf = _lstm_pair(q, 171 + I + H, I, H, s_x)
    Lb, Gb = _lstm_pair(q, 271 + I + H, I, H, s_x)
    x = synth.codes(172 + T + B, (T, B, I), -8, 7)
    need = q.bilstm_layer_workspace(Gf, Gb, T, B)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = host(q.bilstm_layer(Gf, Gb, dev(x), workspace=ws))
    need_f = q.lstm_layer_workspace(Gf, T, B)
    assert q.layer_error_flag(ws, need_f) == 0 and q.layer_error_flag(ws, need) == 0
    assert out.shape == (T, B, 2 * H)
    for d, (L, order) in enumerate(((Lf, range(T)), (Lb, range(T - 1, -1, -1)))):
        hg = out[:, :, d * H:(d + 1) * H]
        hp = np.zeros((B, H), np.int8); cp = np.zeros((B, H), np.float32)
        n_bad = 0
        for t in order:
            hr, cr, dbg = oracle.lstm_step(L, x[t], hp, cp, debug=True)
            assert_codes_close(hg[t], hr, dbg["h_real"] * 7.0, f"dir {d} h t={t}")
            n_bad += int((hg[t] != hr).sum())
            hp, cp = hg[t], cr      # GPU codes forward; cell state from the oracle's step on those codes
        free, _, _, _ = oracle.lstm_layer(L, x, reverse=(d == 1))
        assert (free == hg).mean() >= (1.0 if T * B * H < 5000 else 0.999)


@pytest.mark.parametrize("reverse", [False, True])
def test_lstm_layer_full_size_sampled_steps(gpu_lib, reverse):
    """An encoder layer at its measured size (500 frames x 32 utterances, 1280 -> 640: the launch
    configuration of the persistent recurrence and of the 16000-row input-projection GEMM), checked
    on sampled time steps: one oracle step from the GPU's own state of the step before, plus sampled
    rows of the GEMM, plus the bounded-wait error flag."""
    q = gpu_lib
    T, B, I, H = 500, 32, 1280, 640
    L, G = _lstm_pair(q, 371, I, H, S_H)
    x = synth.codes(372, (T, B, I), -7, 7)
    need = q.lstm_layer_workspace(G, T, B)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    out = q.lstm_layer(G, dev(x), reverse=reverse, want_last=True, debug=True, workspace=ws)
    assert q.layer_error_flag(ws, need) == 0
    hg, cg = host(out["h_out"]), host(out["c_all"])
    rows = np.random.default_rng(373).choice(T * B, 64, replace=False)
    assert np.array_equal(host(out["accx"]).reshape(T * B, 4 * H)[rows], oracle.matmul_i32(L.w_ih, x.reshape(T * B, I)[rows]))
    steps = sorted(np.random.default_rng(374).choice(np.arange(1, T - 1), 6, replace=False).tolist()) + [0, T - 1]
    for t in steps:
        tp = t + 1 if reverse else t - 1            # the step computed before t
        first = (t == T - 1) if reverse else (t == 0)
        hp = np.zeros((B, H), np.int8) if first else hg[tp]
        cp = np.zeros((B, H), np.float32) if first else cg[tp]
        hr, cr, dbg = oracle.lstm_step(L, x[t], hp, cp, debug=True)
        assert_rel(cg[t], cr, f"c t={t}")
        assert_codes_close(hg[t], hr, dbg["h_real"] * 7.0, f"h t={t}")
    last = 0 if reverse else T - 1
    assert np.array_equal(host(out["h_last"]), hg[last]) and np.array_equal(host(out["c_last"]), cg[last])


def test_bilstm_layer_full_size_equals_single_directions(gpu_lib):
    """Both directions in one launch give exactly the codes of the two single-direction calls
    (same kernels, different grouping), at the measured encoder size."""
    q = gpu_lib
    T, B, I, H = 500, 32, 1280, 640
    _, Gf = _lstm_pair(q, 381, I, H, S_H)
    _, Gb = _lstm_pair(q, 391, I, H, S_H)
    x = dev(synth.codes(382, (T, B, I), -7, 7))
    need = q.bilstm_layer_workspace(Gf, Gb, T, B)
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    both = host(q.bilstm_layer(Gf, Gb, x, workspace=ws))
    assert q.layer_error_flag(ws, need) == 0
    f = host(q.lstm_layer(Gf, x)["h_out"])
    b = host(q.lstm_layer(Gb, x, reverse=True)["h_out"])
    assert np.array_equal(both[:, :, :H], f) and np.array_equal(both[:, :, H:], b)


# ------------------------------------------------------------------ joint + fusion, beam

@pytest.mark.parametrize("N,J,V,TB,lms", [(4, 32, 16, 40, True), (1024, 256, 46, 32000, True), (37, 256, 46, 100, True),
                                          (16, 256, 46, 500, False)])
def test_joint_fuse_parity(gpu_lib, N, J, V, TB, lms):
    q = gpu_lib
    e = synth.normal(81 + N, (TB, J), 1.0)
    p = synth.normal(82 + N, (N, J), 1.0)
    fr = np.random.default_rng(83 + N).integers(0, TB, N).astype(np.int32)
    w = synth.normal(84 + N, (V, J), 1.0 / np.sqrt(J) * 3)
    b = synth.normal(85 + N, (V,), 0.1)
    ls = synth.log_probs(86 + N, N, V) if lms else None
    le = synth.log_probs(87 + N, N, V) if lms else None
    out = oracle.Linear.from_float(w, b, S_H)
    m = q.pack_int4(dev(w), q.LAYOUT_TILED)
    fused, lp, zq = q.joint_fuse(dev(e), dev(fr), dev(p), m, dev(b), None if ls is None else dev(ls),
                                 None if le is None else dev(le), 0.3, 0.5, rho=0.2, want_lp=True, want_zq=True)
    zq_r, z_real = oracle.joint_z(e, fr, p, 7.0)
    assert_codes_close(host(zq), zq_r, z_real * 7.0, "z codes")
    # second half from the GPU's own codes: a z tie cannot hide or fake an error downstream
    lp_r, f_r = oracle.joint_out(out, host(zq), ls, le, 0.3, 0.5, rho=0.2, blank=0)
    assert np.abs(host(lp) - lp_r).max() < 1e-3 and np.abs(host(fused) - f_r).max() < 1e-3
    assert np.abs(host(fused) - f_r).max() < 2e-5     # what the arithmetic actually gives
    same = np.all(host(zq) == zq_r, axis=1)
    _, _, f_full = oracle.joint_fuse(e, fr, p, out, ls, le, 0.3, 0.5, rho=0.2)
    assert same.mean() > 0.99 and np.abs(host(fused)[same] - f_full[same]).max() < 1e-3


@pytest.mark.parametrize("B,W,V", [(2, 2, 16), (64, 16, 46), (3, 5, 7), (1, 16, 46)])
def test_beam_step_exact(gpu_lib, B, W, V):
    q = gpu_lib
    rng = np.random.default_rng(91 + B)
    score = rng.standard_normal((B, W)).astype(np.float32) * 3
    fused = synth.log_probs(92 + B, B * W, V)
    if W > 2:
        score[0, W // 2:] = -np.inf                 # dead slots
        score[B - 1, 1:] = -np.inf                  # one live hypothesis only
    fused[0, 1] = fused[0, 3]                       # a tie inside one parent
    if W > 1:
        score[0, 1] = score[0, 0]; fused[1] = fused[0]   # ties across parents
    for force in (False, True):
        got = q.beam_step(dev(score), dev(fused), blank=0, force_blank=force)
        ref = oracle.beam_step(score, fused, blank=0, force_blank=force)
        for g, r, name in zip(got, ref, ("parent", "token", "score")):
            assert np.array_equal(host(g), r), f"{name} force={force}"
