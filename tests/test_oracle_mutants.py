"""Are the oracle's pins sharp?  One plausible mistake at a time (a dropped factor, a wrong index, a
swapped operand, an off-by-one) is planted in a copy of the oracle's source (the C routines, then the
reference blocks that chain them), the copy is rebuilt and the pins are run against it: every mutant has to fail at least one pin.  CPU only; the mistakes
live in temporary copies, never in the tree."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (what goes wrong, text of the oracle, what it becomes); count = occurrences replaced (0 = all)
MUTANTS = [
    ("score_attn without the 1/sqrt(d) scale",
     "z[i] = scale * dot;", "z[i] = dot;", 1),
    ("score_attn with the kv head of a query head taken modulo",
     "const int m = row / Hq, h = row % Hq, hk = h / rep;", "const int m = row / Hq, h = row % Hq, hk = h % Hkv;", 1),
    ("score_attn averaged over text rows only",
     "const double norm = 1.0 / ((double)M * (double)Hq);", "const double norm = 1.0 / ((double)M);", 1),
    ("score_mamba taking the absolute value after the sums",
     "tot += fabs(dot);\n            }\n        s[i] = tot / ((double)M * (double)H);",
     "tot += dot;\n            }\n        s[i] = fabs(tot) / ((double)M * (double)H);", 1),
    ("score_mamba without the step size",
     "dot += (dtv[(size_t)i * H + h] * b[j]) * c[j];", "dot += (b[j]) * c[j];", 1),
    ("score_mamba with heads dealt to groups round-robin",
     "const int g = h / hpg;\n                const double *b = Bv", "const int g = h % G;\n                const double *b = Bv", 1),
    ("decayed score whose decay includes the token's own step",
     "for (int u = i + 1; u <= t; ++u) decay", "for (int u = i; u <= t; ++u) decay", 1),
    ("decayed score whose decay stops one step early",
     "for (int u = i + 1; u <= t; ++u) decay", "for (int u = i + 1; u < t; ++u) decay", 1),
    ("selection of the K lowest scores",
     "for (int r = 0; r < K; ++r) idx[r] = p[r].i;", "for (int r = 0; r < K; ++r) idx[r] = p[N - 1 - r].i;", 1),
    ("selection left in score order",
     "qsort(idx, (size_t)K, sizeof(int32_t), cmp_index_asc);", "", 1),
    ("compaction taking the text rows from row K on",
     "sp + (size_t)(N + m) * row_bytes", "sp + (size_t)(K + m) * row_bytes", 1),
    ("compaction that forgets earlier position maps",
     "pos_out[r] = pos_in ? pos_in[idx[r]] : idx[r];", "pos_out[r] = idx[r];", 1),
    ("recurrence without the step size on the input",
     "+ xt[p] * (dtt * b[j]);", "+ xt[p] * (b[j]);", 1),
    ("recurrence reading the state before updating it",
     "S[(size_t)p * n + j] = a * S[(size_t)p * n + j] + xt[p] * (dtt * b[j]);\n"
     "                    out += S[(size_t)p * n + j] * c[j];",
     "out += S[(size_t)p * n + j] * c[j];\n"
     "                    S[(size_t)p * n + j] = a * S[(size_t)p * n + j] + xt[p] * (dtt * b[j]);", 1),
    ("recurrence with a decay that ignores the step size",
     "const double a = exp(dtt * A[h]);", "const double a = exp(A[h]);", 1),
    ("recurrence with b and c exchanged",
     "const double *b = B + ((size_t)t * G + g) * n;\n            const double *c = C + ((size_t)t * G + g) * n;\n"
     "            const double *xt",
     "const double *b = C + ((size_t)t * G + g) * n;\n            const double *c = B + ((size_t)t * G + g) * n;\n"
     "            const double *xt", 1),
    ("unrolled form whose decay includes step j",
     "for (int u = j + 1; u <= t; ++u) decay", "for (int u = j; u <= t; ++u) decay", 1),
    ("unrolled form whose initial state misses the first decay",
     "for (int u = 0; u <= t; ++u) decay", "for (int u = 1; u <= t; ++u) decay", 1),
    ("chunked form that carries the state without decay",
     "Sn[e] = exp(l[Q - 1]) * S[e];", "Sn[e] = S[e];", 1),
    ("chunked form with the wrong sign in the intra-chunk decay",
     "const double w = exp(l[t] - l[j]) * cb", "const double w = exp(l[j] - l[t]) * cb", 1),
    ("attention without the diagonal",
     "for (int j = 0; j <= t; ++j) {\n                const double *kv", "for (int j = 0; j < t; ++j) {\n                const double *kv", 1),
    ("attention with the kv head of a query head taken modulo",
     "const int hk = h / rep;\n            const double *qv = q + ((size_t)t", "const int hk = h % Hkv;\n            const double *qv = q + ((size_t)t", 1),
    ("rmsnorm with eps outside the root",
     "const double inv = 1.0 / sqrt(ss / d + eps);", "const double inv = 1.0 / (sqrt(ss / d) + eps);", 1),
    ("gated norm with the gate on the wrong operand",
     "y[o + c] * oracle_silu(z[o + c])", "oracle_silu(y[o + c]) * z[o + c]", 0),
    ("gated norm normalised over all channels at once",
     "const double inv = 1.0 / sqrt(ss / gs + eps);", "const double inv = 1.0 / sqrt(ss / D + eps);", 1),
    ("convolution with the taps reversed",
     "acc += w[(size_t)c * W + k] * in", "acc += w[(size_t)c * W + (W - 1 - k)] * in", 1),
    ("convolution that looks ahead",
     "const int ts = t - (W - 1) + k;\n                if (ts >= 0)", "const int ts = t + k;\n                if (ts < T)", 1),
    ("softplus without the bias",
     "+ (bias ? bias[h] : 0.0);", "+ 0.0;", 1),
    ("pooling windows rounded up",
     "hi = (int)(((long long)(j + 1) * N) / K);", "hi = (int)(((long long)(j + 1) * N + K - 1) / K);", 1),
    ("pooled token placed at the end of its window",
     "pos_out[j] = pos_in ? pos_in[lo] : lo;", "pos_out[j] = pos_in ? pos_in[hi - 1] : hi - 1;", 1),
    ("equal scores resolved towards the higher index",
     "return (x->i > y->i) - (x->i < y->i);", "return (x->i < y->i) - (x->i > y->i);", 1),
    ("recurrence without the skip term",
     "yt[p] = out + (D ? D[h] * xt[p] : 0.0);", "yt[p] = out;", 1),
    ("recurrence that ignores the incoming state",
     "if (S_in) memcpy(S, S_in + (size_t)h * P * n, sizeof(double) * (size_t)P * n);\n        for (int t = 0; t < T; ++t) {\n"
     "            const double dtt",
     "for (int t = 0; t < T; ++t) {\n            const double dtt", 1),
    ("recurrence that hands the state back in another head's slot",
     "if (S_out) memcpy(S_out + (size_t)h * P * n, S, sizeof(double) * (size_t)P * n);\n        free(S);\n    }",
     "if (S_out) memcpy(S_out + (size_t)(H - 1 - h) * P * n, S, sizeof(double) * (size_t)P * n);\n        free(S);\n    }", 1),
    ("decayed score with growth instead of decay",
     "decay *= exp(dt[(size_t)u * H + h] * A[h]);\n                const double *b = Ball",
     "decay *= exp(-dt[(size_t)u * H + h] * A[h]);\n                const double *b = Ball", 1),
    ("convolution without the bias",
     "double acc = b ? b[c] : 0.0;", "double acc = 0.0;", 1),
    ("pooling that averages the text rows in",
     "dst[(size_t)(K + m) * D + c] = src[(size_t)(N + m) * D + c];", "dst[(size_t)(K + m) * D + c] = src[(size_t)(N - 1) * D + c];", 1),
    ("softmax attention normalised by the largest weight",
     "const double w = z[j] / denom;", "const double w = z[j];", 1),
]

# and for the thin Python layer over the C routines (oracle/__init__.py)
WRAPPER_MUTANTS = [
    ("default scale 1/d instead of 1/sqrt(d)",
     "scale = 1.0 / np.sqrt(d)", "scale = 1.0 / d", 0),
    ("decode step that queries with the oldest row",
     "q[T - 1] = q1\n    return attn(q, k, v, scale=scale, rows=[T - 1])[0]", "q[0] = q1\n    return attn(q, k, v, scale=scale, rows=[0])[0]", 1),
]

# the same for the reference blocks (oracle/blocks.py), which chain the oracle's routines
BLOCK_MUTANTS = [
    ("block with B and C taken from each other's columns",
     "xbc[:, d_inner:d_inner + gn].reshape(T, G, n), \\\n        xbc[:, d_inner + gn:].reshape(T, G, n)",
     "xbc[:, d_inner + gn:].reshape(T, G, n), \\\n        xbc[:, d_inner:d_inner + gn].reshape(T, G, n)", 1),
    ("block without the residual connection",
     "return r(g @ wt[\"W_out\"] + hidden), pre", "return r(g @ wt[\"W_out\"]), pre", 1),
    ("block whose gated norm runs over all channels at once",
     "wt[\"gnorm_w\"], G, eps)", "wt[\"gnorm_w\"], 1, eps)", 1),
    ("block without the dt bias",
     "softplus_dt(xbcdt[:, d_inner + 2 * gn:], wt[\"dt_bias\"])", "softplus_dt(xbcdt[:, d_inner + 2 * gn:], None)", 1),
    ("reduced block that forgets to compact the gate",
     "x, B, C, dt, z, hidden = (compact(a, idx, N, M)[0] for a in (x, B, C, dt, z, hidden))",
     "x, B, C, dt, hidden = (compact(a, idx, N, M)[0] for a in (x, B, C, dt, hidden)); z = z[:idx.shape[0] + M]", 1),
    ("attention block that compacts the wrong residual rows",
     "q, k, v, hidden = (compact(a, idx, N, M)[0] for a in (q, k, v, hidden))",
     "q, k, v = (compact(a, idx, N, M)[0] for a in (q, k, v)); hidden = hidden[:idx.shape[0] + M]", 1),
    ("attention block with keys from the value projection",
     "k = r(u @ wt[\"W_k\"]).reshape(T, Hkv, d)", "k = r(u @ wt[\"W_v\"]).reshape(T, Hkv, d)", 1),
]


def _run_mutant(args):
    slot, (what, old, new, count), (fname, source), base = args
    d = os.path.join(base, "m%d" % slot)
    shutil.rmtree(d, ignore_errors=True)
    os.makedirs(os.path.join(d, "oracle"))
    for name in ("__init__.py", "blocks.py", "strd_oracle.c"):
        shutil.copy(os.path.join(ROOT, "oracle", name), os.path.join(d, "oracle", name))
    with open(os.path.join(d, "oracle", fname), "w") as fh:
        fh.write(source.replace(old, new) if count == 0 else source.replace(old, new, count))
    shutil.copytree(os.path.join(ROOT, "tests"), os.path.join(d, "tests"), ignore=shutil.ignore_patterns("__pycache__"))
    os.symlink(os.path.join(ROOT, "paper_2603_00198_amd"), os.path.join(d, "paper_2603_00198_amd"))
    env = dict(os.environ, OMP_NUM_THREADS="2", PYTHONDONTWRITEBYTECODE="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=d, env=env, capture_output=True, text=True, timeout=600)
    return what, r.returncode, r.stdout[-600:]


def _source(fname):
    with open(os.path.join(ROOT, "oracle", fname)) as fh:
        return fname, fh.read()


def test_every_planted_mistake_fails_a_pin(tmp_path):
    jobs = [(m, _source("strd_oracle.c")) for m in MUTANTS] + [(m, _source("blocks.py")) for m in BLOCK_MUTANTS] + \
        [(m, _source("__init__.py")) for m in WRAPPER_MUTANTS]
    for (what, old, new, count), (fname, source) in jobs:
        assert old in source, "%s no longer contains the text this mutant replaces: %s" % (fname, what)
    workers = 4
    survivors, broken = [], []
    for start in range(0, len(jobs), workers):
        batch = [(slot, m, src, str(tmp_path)) for slot, (m, src) in enumerate(jobs[start:start + workers])]
        with ThreadPoolExecutor(workers) as pool:
            for what, rc, tail in pool.map(_run_mutant, batch):
                if rc == 0:
                    survivors.append(what)
                elif rc != 1:                      # 1 = tests ran and some failed; anything else is a broken run
                    broken.append((what, rc, tail))
    assert not broken, "mutant runs that did not get as far as a failing pin: %r" % (broken,)
    assert not survivors, "no pin notices: " + "; ".join(survivors)


def test_the_unchanged_oracle_passes_in_the_same_harness(tmp_path):
    """The harness itself: the same copy-build-run with nothing planted passes."""
    what, rc, tail = _run_mutant((0, ("nothing", "", "", 1), _source("strd_oracle.c"), str(tmp_path)))
    assert rc == 0, tail
