"""Do the pins bite?  Each case plants one plausible mistake in a private copy of the
oracle's C source (a dropped term, a wrong sign, index, bound or rounding), rebuilds that
copy with gcc and runs tests/test_oracle_pins.py against it in a child process: the pins
must fail.  The unmodified copy must pass.  CPU only; the GPU path is not involved.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in oracle/qrnnt_oracle.c, replacement).  The text must occur exactly once.
MUTANTS = [
    ("quantizer rounds half up instead of to even",
     "    float r = nearbyintf(t); /* default rounding mode: ties to even */", "    float r = floorf(t + 0.5f);"),
    ("quantizer truncates", "    float r = nearbyintf(t);\n    if (r < lo) r = lo;", "    float r = truncf(t);\n    if (r < lo) r = lo;"),
    ("upper clamp at 8", "    if (r > 7.0f) r = 7.0f;", "    if (r > 8.0f) r = 8.0f;"),
    ("b-bit clamp one code too wide", "hi = (float)((1 << (bits - 1)) - 1);", "hi = (float)(1 << (bits - 1));"),
    ("weight step alpha/8", "        float s = alpha / 7.0f;", "        float s = alpha / 8.0f;"),
    ("g gate through a sigmoid", "double gg = tanh(pre[2 * H + j]);", "double gg = sigm(pre[2 * H + j]);"),
    ("forget and output gates swapped",
     "            double gf = sigm(pre[H + j]);\n            double gg = tanh(pre[2 * H + j]);\n            double go = sigm(pre[3 * H + j]);",
     "            double gf = sigm(pre[3 * H + j]);\n            double gg = tanh(pre[2 * H + j]);\n            double go = sigm(pre[H + j]);"),
    ("cell update without the forget gate", "double c = gf * (double)cp[j] + gi * gg;", "double c = (double)cp[j] + gi * gg;"),
    ("hidden state without tanh", "double h = go * tanh(c);", "double h = go * c;"),
    ("parent gather ignored", "int src = parent ? parent[n] : n;", "int src = n;"),
    ("recurrent part scaled by the input rows' steps",
     "(double)L->s_h * (double)L->s_whh[r] * (double)ah", "(double)L->s_h * (double)L->s_wih[r] * (double)ah"),
    ("LSTM bias dropped", "(double)ah + (double)L->bias[r];", "(double)ah;"),
    ("reverse direction walks forward", "int t = reverse ? T - 1 - s : s;", "int t = s;"),
    ("additive joint", "double z = tanh((double)e[j] * (double)p[j]);", "double z = tanh((double)e[j] + (double)p[j]);"),
    ("source LM added instead of subtracted", "f -= (double)lambda_src *", "f += (double)lambda_src *"),
    ("external LM subtracted", "f += (double)lambda_ext *", "f -= (double)lambda_ext *"),
    ("label reward dropped", "                f += (double)rho;\n", ""),
    ("log-softmax without the max shift restored", "lp[k] = x[k] - m - ls;", "lp[k] = x[k] - ls;"),
    ("last index wins a tie in the beam step", "if (best < 0 || val[c] > val[best]) best = c;", "if (best < 0 || val[c] >= val[best]) best = c;"),
    ("labels allowed in the last round of a frame", "beam_step_core(S, F, 1, W, V, M->blank, v == max_sym, par, tk, ns, want ? &sm : NULL);",
     "beam_step_core(S, F, 1, W, V, M->blank, 0, par, tk, ns, want ? &sm : NULL);"),
    ("blank keeps the old score", "                        Nx[nNx].score = ns[r];\n", ""),
    ("linear layer bias dropped", "(double)s + (P->bias ? (double)P->bias[r] : 0.0);", "(double)s;"),
    ("a blank pick copies the wrong hypothesis", "hyp_copy(M, &Nx[nNx], &A[par[r]]);", "hyp_copy(M, &Nx[nNx], &A[r < nA ? r : 0]);"),
    ("the frame's pruning keeps the worst", "if (best < 0 || Nx[i].score > Nx[best].score) best = i;",
     "if (best < 0 || Nx[i].score < Nx[best].score) best = i;"),
    ("nibbles packed high first", "(uint8_t)((lo & 0xF) | ((hi & 0xF) << 4));", "(uint8_t)((hi & 0xF) | ((lo & 0xF) << 4));"),
    ("b-bit weight step alpha/2^(b-1)", "        scale[r] = alpha / qmax;", "        scale[r] = alpha / (qmax + 1.0f);"),
    ("ALSD: recombination keeps the maximum", "const float sc = (float)(m + log(sum));", "const float sc = (float)m;"),
    ("ALSD: every hypothesis reads frame i", "int t = live ? i - cur[w].len : 0;", "int t = live ? i : 0;"),
    ("ALSD: one label more than the cap", "if (cur[w].len >= u_max)", "if (cur[w].len > u_max)"),
    ("ALSD: finishing blank stays a candidate", "                    F[(int64_t)w * V + M->blank] = -INFINITY;\n", ""),
    ("bottleneck output not quantized to the grid", "oq_quantize_sym(ym, net->mid.rows, net->inv_s_mid, net->out.bits, qm);",
     "for (int q = 0; q < net->mid.rows; ++q) qm[q] = (int8_t)(ym[q] * net->inv_s_mid);"),
    ("upper LSTM layers of a network see zero state from the layer below",
     "        memcpy(xin, dst->h[l], (size_t)net->layer[l].H);", "        memset(xin, 0, (size_t)maxw);"),
    ("a layer's initial cell state ignored", "    if (c0) memcpy(c, c0, (size_t)B * H * sizeof(float));\n", ""),
    ("a layer's initial hidden codes ignored", "    if (h0) memcpy(h, h0, (size_t)B * H);\n", ""),
    ("tie distance taken on the fp64 product", "const double t = (double)(x * inv_s);", "const double t = (double)x * (double)inv_s;"),
    ("tie distance on the 8-bit grid not scaled to 4-bit steps", "return fabs(frac - 0.5) * (7.0 / qmax);", "return fabs(frac - 0.5);"),
    ("clamped values counted as near ties", "    if (t <= -qmax - 1.5 || t >= qmax + 0.5) return INFINITY;\n", ""),
    ("selection gap ignores the best candidate left out", "            for (int r = 0; r <= W; ++r) {", "            for (int r = 0; r < W; ++r) {"),
    ("margin of the start-symbol advance dropped", "hyp_extend(M, &beam[0], &zero, 0, 0.0f, want ? &qm : NULL);",
     "hyp_extend(M, &beam[0], &zero, 0, 0.0f, NULL);"),
    ("ALSD: margin of the start-symbol advance dropped", "hyp_extend(M, &cur[0], &zero, 0, 0.0f, want ? &qm : NULL);",
     "hyp_extend(M, &cur[0], &zero, 0, 0.0f, NULL);"),
    ("cache: a hit in the beam takes the parent's own sequence for the new one",
     "same_seq(cur[j].tok, cur[j].len, pr->tok, pr->len, tk[r])) hit = &cur[j];",
     "same_seq(cur[j].tok, cur[j].len, pr->tok, pr->len, -1)) hit = &cur[j];"),
    ("cache: extended sequences are never remembered", "cache_ent *ce = &cache[n_cache++];", "cache_ent *ce = &cache[n_cache]; n_cache += 0;"),
    ("cache: sequences compared by length only", "        if (a[p] != (p < lb ? b[p] : extra_b)) return 0;\n", ""),
    ("z decisions not counted in the margin", "for (int w = 0; w < nA; ++w) if (rowm[w] < qm) qm = rowm[w];",
     "for (int w = 0; w < nA; ++w) if (rowm[w] < 0.0) qm = rowm[w];"),
]

FILES = ["oracle", "tests/test_oracle_pins.py", "tests/conftest.py", "tests/golden", "paper_2206_07882_amd/synth.py",
         "paper_2206_07882_amd/__init__.py"]


def _run(tmp, idx, name, old, new):
    d = os.path.join(tmp, "m%03d" % idx)
    for rel in FILES:
        src, dst = os.path.join(ROOT, rel), os.path.join(d, rel)
        os.makedirs(os.path.dirname(dst), exist_ok=True)
        if os.path.isdir(src):
            shutil.copytree(src, dst, ignore=shutil.ignore_patterns("*.so", "__pycache__"))
        else:
            shutil.copy(src, dst)
    path = os.path.join(d, "oracle", "qrnnt_oracle.c")
    text = open(path).read()
    if old is not None:
        assert text.count(old) == 1, f"mutation site of '{name}' occurs {text.count(old)} times"
        open(path, "w").write(text.replace(old, new))
    env = dict(os.environ, PYTHONPATH=d, OMP_NUM_THREADS="1", PYTHONDONTWRITEBYTECODE="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=d, env=env, capture_output=True, text=True, timeout=600)
    return name, r.returncode, (r.stdout + r.stderr)[-600:]


def test_pins_catch_planted_mistakes(tmp_path):
    jobs = [("unmodified", None, None)] + MUTANTS
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda ij: _run(str(tmp_path), ij[0], *ij[1]), enumerate(jobs)))
    name, rc, tail = results[0]
    assert rc == 0, "the pins fail on an unmodified copy of the oracle:\n" + tail
    survivors = [n for n, rc, _ in results[1:] if rc == 0]
    assert not survivors, "no pin notices: " + "; ".join(survivors)
    broken = [(n, t) for n, rc, t in results[1:] if rc not in (0, 1)]   # 1 = tests failed; anything else = could not run
    assert not broken, "mutant runs that did not get as far as the pins: " + repr(broken)
