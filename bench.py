#!/usr/bin/env python3
"""Benchmark of the token-reduced prefill of one hybrid layer on one MI355X.

A step is one pass of the whole hot path over one synthetic long-video-shaped sequence:
score -> select_topk -> compact (every mixer input + the hidden states) -> mixer on the K + M
survivors, all enqueued on one HIP stream without host synchronisation.  Inputs are resident
in HBM before the timed region.  One JSON line is printed.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5m|c5a|c2|c3|c4m|c4a]
                  [--budget 0.25] [--no-cpu-baseline] [--no-extras]

The default line is the long-video configuration (131072 vision + 512 text tokens, 25 %): the
Mamba-2 layer is `value`, the attention layer of the same configuration rides along under
`attention_layer` with the same steps and warm-up, the two smaller single-layer workloads under
`other_workloads`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
KERNEL_STEP = 64               # tokens per step of the scan kernel, whatever `chunk` the caller names
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.md")


def source_hash(file_name):
    import hashlib
    path = os.path.join(ROOT, "paper_2603_00198_amd", "csrc", file_name)
    try:
        return hashlib.sha1(open(path, "rb").read()).hexdigest()[:12]
    except OSError:
        return None


def measured_traffic(workload, budget, kernel):
    """HBM bytes per launch of the mixer kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE counter runs
    summarised in profiles/hbm_traffic.md (counters cannot be read from inside this process).  A row
    names the source file of the kernel that was profiled and counts only while that file is unchanged;
    otherwise None."""
    try:
        rows = open(TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None
    for line in rows:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 7 and cells[0] == workload and cells[2] == kernel:
            try:
                if abs(float(cells[1]) - budget) > 1e-9 or cells[6] != source_hash(cells[3]):
                    continue
                return float(cells[4]) + float(cells[5])
            except ValueError:
                continue
    return None


PAPER_CONTEXT = "paper: 3.8-4.2x LLM-stage prefill speed-up at ~25% budget, whole 12B hybrid, 1x A100, 36864 vision tokens"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5m",
                    help="headline workload (default c5m: the Mamba-2 layer of the long-video configuration, the "
                         "largest one; the line then also carries c5a, c2 and c3)")
    ap.add_argument("--budget", type=float, default=0.25)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile", action="store_true",
                    help="for rocprofv3: only the warm-up and the timed reduced steps, then one plain copy of "
                         "known size (256 MiB through the compact kernel with the identity index list) that "
                         "calibrates the FETCH_SIZE / WRITE_SIZE counters; prints the byte counts")
    ap.add_argument("--stack-model", action="store_true",
                    help="instead of the layer benchmark: measure the Mamba-2 and attention layer at every token "
                         "count the paper's named schedules visit (c4 shapes) and print the modelled speed-up of "
                         "the mixers of the 62-layer hybrid under each schedule")
    ap.add_argument("--variants", action="store_true",
                    help="time only the average-pool baseline and the decode steps (next_rows.variants of the default line)")
    ap.add_argument("--batch", type=int, default=0,
                    help="run this many independent sequences of the workload on one stream each and report the aggregate rate")
    ap.add_argument("--block-stack", action="store_true",
                    help="instead of the layer benchmark: the 8-block hidden-to-hidden stack of workload c4 "
                         "(projections, glue, mixers, residual) with the progressive budgets against the same "
                         "stack without reduction")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline workload: skip the other layers appended to the default line")
    return ap.parse_args()


WORKLOADS = {           # name -> (synth workload, layer kind)
    "c2": ("c2", "mamba"), "c3": ("c3", "attn"), "c4m": ("c4", "mamba"), "c4a": ("c4", "attn"),
    "c5m": ("c5", "mamba"), "c5a": ("c5", "attn"),
}


class EventPairs:
    """HIP event pairs recorded on torch's current stream (the stream the library launches on)."""

    def __init__(self, torch):
        self.torch, self.pairs = torch, []

    def wrap(self, fn):
        a = self.torch.cuda.Event(enable_timing=True)
        b = self.torch.cuda.Event(enable_timing=True)
        a.record()
        out = fn()
        b.record()
        self.pairs.append((a, b))
        return out

    def mean_ms(self):
        return sum(a.elapsed_time(b) for a, b in self.pairs) / max(len(self.pairs), 1)


def time_loop(torch, fn, steps, warmup):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_events(torch, fn, iters=20, warmup=3):
    for _ in range(warmup):
        fn()
    ev = EventPairs(torch)
    for _ in range(iters):
        ev.wrap(fn)
    torch.cuda.synchronize()
    return ev.mean_ms()


def time_graph(torch, fn, reps=20, replays=5):
    """Mean ms per call of `fn` with `reps` calls captured into one HIP graph and replayed: the
    device time of kernels that are shorter than the host's launch path."""
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(reps):
                fn()
    torch.cuda.current_stream().wait_stream(side)
    graph.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * reps)


class MambaLayer:
    kind = "mamba"

    def __init__(self, torch, strd, synth, w, dev):
        self.torch, self.strd, self.w = torch, strd, w
        s = w.mamba
        self.s = s
        N, M, K = w.N, w.M, w.K
        hidden = synth.hidden_states(w, dev)
        t = synth.mamba_inputs(w, hidden)
        self.hidden = hidden.to(synth.torch_dtype(w.dtype))
        self.t = t
        self.Bv = t["B"][:N].contiguous(); self.Ct = t["C"][N:].contiguous(); self.dtv = t["dt"][:N].contiguous()
        e = lambda *shape, dtype=self.hidden.dtype: torch.empty(*shape, dtype=dtype, device=dev)
        self.scores = e(N, dtype=torch.float32)
        self.idx = e(K, dtype=torch.int32)
        Tr = K + M
        self.o = {"x": e(Tr, s.H, s.P), "B": e(Tr, s.G, s.n), "C": e(Tr, s.G, s.n),
                  "dt": e(Tr, s.H, dtype=torch.float32), "hidden": e(Tr, w.d_model)}
        self.fused = False   # True: ssd_prefill_gather reads x, dt, B, C through idx; only hidden is compacted
        self.y_red = e(Tr, s.H, s.P)
        self.y_full = e(w.T, s.H, s.P)
        lib = strd.lib()
        io = 1 if w.dtype == "bf16" else 0
        nb = max(lib.strd_score_mamba_workspace(M, N, s.H, s.G, s.n, io),
                 lib.strd_ssd_prefill_workspace(w.T, s.H, s.P, s.G, s.n, s.chunk, io),
                 lib.strd_select_topk_workspace(N, w.K), 16)
        self.ws = e(nb, dtype=torch.uint8)
        self.ws_full = e(max(lib.strd_score_mamba_full_workspace(M, N, s.H, s.G, s.n, io), 16), dtype=torch.uint8)
        self.scores_full = e(N, dtype=torch.float32)
        self.mixer_ev = None

    def score(self):
        self.strd.score_mamba(self.Bv, self.Ct, self.dtv, out=self.scores, ws=self.ws)

    def score_full(self):   # the Full Mamba Dynamic score (ablation row), not part of the step
        self.strd.score_mamba_full(self.Bv, self.Ct, self.t["dt"], self.t["A"], out=self.scores_full, ws=self.ws_full)

    def select(self):
        self.strd.select_topk(self.scores, self.w.K, out=self.idx, ws=self.ws)

    def compact(self):
        N, M = self.w.N, self.w.M
        if self.fused:   # the scan reads its inputs through the index list, so only the residual stream moves
            self.strd.compact_batch([self.hidden], self.idx, N, M, outs=[self.o["hidden"]])
            return
        keys = ("x", "B", "C", "dt")
        self.strd.compact_batch([self.t[k] for k in keys] + [self.hidden], self.idx, N, M,
                                outs=[self.o[k] for k in keys] + [self.o["hidden"]])

    def mixer_reduced(self):
        t, o = self.t, self.o
        if self.fused:
            self.strd.ssd_prefill_gather(t["x"], t["dt"], t["A"], t["B"], t["C"], self.idx, self.w.N, self.w.M,
                                         chunk=self.s.chunk, want_state=False, out=self.y_red, ws=self.ws)
        else:
            self.strd.ssd_prefill(o["x"], o["dt"], t["A"], o["B"], o["C"], chunk=self.s.chunk, want_state=False,
                                  out=self.y_red, ws=self.ws)

    def mixer_full(self):
        t = self.t
        self.strd.ssd_prefill(t["x"], t["dt"], t["A"], t["B"], t["C"], chunk=self.s.chunk, want_state=False,
                              out=self.y_full, ws=self.ws)

    def step(self):
        self.score(); self.select(); self.compact()
        if self.mixer_ev is not None:
            self.mixer_ev.wrap(self.mixer_reduced)
        else:
            self.mixer_reduced()

    # algorithmic HBM bytes / flops of the mixer on T tokens
    def mixer_bytes(self, T):
        s, eb = self.s, self.hidden.element_size()
        return T * (2 * s.H * s.P * eb + 2 * s.G * s.n * eb + 4 * s.H)

    def mixer_flops(self, T, Q=KERNEL_STEP):
        """Causal flop count of the chunked scan with intra-chunk length Q: Q = 64 is what the kernel's
        formulation needs (its step length), Q = the workload's chunk the count of that formulation."""
        s = self.s
        return T * (s.H * (Q * s.P + 4 * s.n * s.P) + s.G * Q * s.n)

    def compact_bytes(self):
        w, s, eb = self.w, self.s, self.hidden.element_size()
        row = w.d_model * eb if self.fused else (s.H * s.P + 2 * s.G * s.n + w.d_model) * eb + 4 * s.H
        return 2 * (w.K + w.M) * row + 4 * w.K * (1 if self.fused else 5)

    def score_work(self):   # (algorithmic bytes, flops) of score_mamba
        w, s, eb = self.w, self.s, self.hidden.element_size()
        return (w.N * (s.G * s.n * eb + 4 * s.H) + w.M * s.G * s.n * eb + 4 * w.N, 2.0 * w.M * w.N * s.n * s.G)

    mixer_name, mixer_bound = "ssd_prefill", "hbm"


class AttnLayer:
    kind = "attn"

    def __init__(self, torch, strd, synth, w, dev):
        self.torch, self.strd, self.w = torch, strd, w
        s = w.attn
        self.s = s
        N, M, K = w.N, w.M, w.K
        hidden = synth.hidden_states(w, dev)
        self.t = synth.attn_inputs(w, hidden)
        self.hidden = hidden.to(synth.torch_dtype(w.dtype))
        self.qt = self.t["q"][N:].contiguous(); self.kv = self.t["k"][:N].contiguous()
        e = lambda *shape, dtype=self.hidden.dtype: torch.empty(*shape, dtype=dtype, device=dev)
        self.scores = e(N, dtype=torch.float32)
        self.idx = e(K, dtype=torch.int32)
        Tr = K + M
        self.o = {"q": e(Tr, s.Hq, s.d), "k": e(Tr, s.Hkv, s.d), "v": e(Tr, s.Hkv, s.d), "hidden": e(Tr, w.d_model)}
        self.o_red = e(Tr, s.Hq, s.d)
        self.o_full = e(w.T, s.Hq, s.d)
        lib = strd.lib()
        io = 1 if w.dtype == "bf16" else 0
        nb = max(lib.strd_score_attn_workspace(M, N, s.Hq, s.Hkv, s.d, io),
                 lib.strd_attn_prefill_workspace(w.T, s.Hq, s.Hkv, s.d, io),
                 lib.strd_select_topk_workspace(N, w.K), 16)
        self.ws = e(nb, dtype=torch.uint8)
        self.mixer_ev = None

    def score(self):
        self.strd.score_attn(self.qt, self.kv, out=self.scores, ws=self.ws)

    def select(self):
        self.strd.select_topk(self.scores, self.w.K, out=self.idx, ws=self.ws)

    def compact(self):
        N, M = self.w.N, self.w.M
        keys = ("q", "k", "v")
        self.strd.compact_batch([self.t[k] for k in keys] + [self.hidden], self.idx, N, M,
                                outs=[self.o[k] for k in keys] + [self.o["hidden"]])

    def mixer_reduced(self):
        o = self.o
        self.strd.attn_prefill(o["q"], o["k"], o["v"], out=self.o_red, ws=self.ws)

    def mixer_full(self):
        t = self.t
        self.strd.attn_prefill(t["q"], t["k"], t["v"], out=self.o_full, ws=self.ws)

    def step(self):
        self.score(); self.select(); self.compact()
        if self.mixer_ev is not None:
            self.mixer_ev.wrap(self.mixer_reduced)
        else:
            self.mixer_reduced()

    def mixer_bytes(self, T):
        s, eb = self.s, self.hidden.element_size()
        return T * (2 * s.Hq * s.d + 2 * s.Hkv * s.d) * eb

    def mixer_flops(self, T, Q=None):
        s = self.s
        return 2.0 * T * T * s.d * s.Hq          # causal: half of 4 T^2 d Hq

    def compact_bytes(self):
        w, s, eb = self.w, self.s, self.hidden.element_size()
        row = (s.Hq * s.d + 2 * s.Hkv * s.d + w.d_model) * eb
        return 2 * (w.K + w.M) * row + 4 * w.K * 4

    def score_work(self):   # (algorithmic bytes, flops by definition -- executed twice) of score_attn
        w, s, eb = self.w, self.s, self.hidden.element_size()
        return (w.N * s.Hkv * s.d * eb + w.M * s.Hq * s.d * eb + 4 * w.N, 2.0 * w.M * w.N * s.d * s.Hq)

    mixer_name, mixer_bound = "attn_prefill", "mfma"


def cpu_baseline_mamba(layer, synth, budget_s=12.0):
    """The fp64 oracle, as it stands, on the same reduced Mamba-2 layer.  Short sequences: all of it,
    repeated for about `budget_s` seconds.  Long ones: score, selection and compaction in full, the scan
    on two heads of every group (heads are independent; the time is scaled to all heads)."""
    import numpy as np
    import oracle
    w, t, s = layer.w, layer.t, layer.s
    N, M, K = w.N, w.M, w.K
    f = synth.np64
    small = N <= 20000
    heads = list(range(s.H)) if small else sorted({g * (s.H // s.G) + j for g in range(s.G) for j in (0, 1)} & set(range(s.H)))
    hsel = layer.torch.tensor(heads, device=t["x"].device)
    Bv, Ct, dtv = f(t["B"][:N]), f(t["C"][N:]), f(t["dt"][:N])
    full = {"x": f(t["x"][:, hsel]), "dt": f(t["dt"][:, hsel]), "B": f(t["B"]), "C": f(t["C"])}
    A = f(t["A"][hsel])
    grp = np.array([h // (s.H // s.G) for h in heads])
    hid = layer.hidden.cpu().view(layer.torch.int16).numpy() if w.dtype == "bf16" else layer.hidden.cpu().numpy()
    oracle.select_topk(np.zeros(4), 2)          # load the library outside the timed region
    reps, t_rest, t_scan, t0 = 0, 0.0, 0.0, time.perf_counter()
    while reps < 40 and time.perf_counter() - t0 < budget_s:
        ta = time.perf_counter()
        sc = oracle.score_mamba(Bv, Ct, dtv)
        idx = oracle.select_topk(sc, K)
        red = {k: oracle.compact(v, idx, N, M)[0] for k, v in full.items()}
        oracle.compact(hid, idx, N, M)
        tb = time.perf_counter()
        if small:
            oracle.ssd_seq(red["x"], red["dt"], A, red["B"], red["C"])
        else:   # one call per group: its two sampled heads against the group's B, C
            for g in range(s.G):
                sel = np.nonzero(grp == g)[0]
                oracle.ssd_seq(red["x"][:, sel], red["dt"][:, sel], A[sel], red["B"][:, g:g + 1], red["C"][:, g:g + 1])
        tc = time.perf_counter()
        t_rest += tb - ta
        t_scan += tc - tb
        reps += 1
    dt = (t_rest + t_scan * (s.H / len(heads))) / reps
    what = ("the whole reduced layer of this workload (all %d vision + %d text tokens, all heads), fp64, mean of %d "
            "passes of %.2f s" % (N, M, reps, dt)) if small else (
            "score, selection and compaction of all %d + %d tokens in full (%.1f s), the scan over the %d survivors on "
            "%d of %d heads (%.1f s), scaled to all heads: est. %.1f s for the whole layer; x was compacted for the "
            "sampled heads only" % (N, M, t_rest / reps, K + M, len(heads), s.H, t_scan / reps, dt))
    return {"value": (N + M) / dt, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle", "sample": what}


def cpu_single_thread_c1(torch, synth):
    """The oracle on the whole tiny pair c1 (reduced Mamba-2 layer + reduced attention layer) with one thread."""
    import subprocess
    code = (
        "import time, numpy as np, torch, oracle\n"
        "from paper_2603_00198_amd import synth\n"
        "w = synth.WORKLOADS['c1']; N, M, K = w.N, w.M, w.K; f = synth.np64\n"
        "h = synth.hidden_states(w, 'cpu'); t = synth.mamba_inputs(w, h); a = synth.attn_inputs(w, h)\n"
        "oracle.select_topk(np.zeros(4), 2)\n"
        "t0 = time.perf_counter()\n"
        "s = oracle.score_mamba(f(t['B'][:N]), f(t['C'][N:]), f(t['dt'][:N])); i = oracle.select_topk(s, K)\n"
        "r = {k: oracle.compact(f(t[k]), i, N, M)[0] for k in ('x', 'dt', 'B', 'C')}\n"
        "oracle.ssd_seq(r['x'], r['dt'], f(t['A']), r['B'], r['C'])\n"
        "s = oracle.score_attn(f(a['q'][N:]), f(a['k'][:N])); i = oracle.select_topk(s, K)\n"
        "r = {k: oracle.compact(f(a[k]), i, N, M)[0] for k in ('q', 'k', 'v')}\n"
        "oracle.attn(r['q'], r['k'], r['v'])\n"
        "print(time.perf_counter() - t0)\n")
    env = dict(os.environ, OMP_NUM_THREADS="1")
    out = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=300,
                         cwd=os.path.dirname(os.path.abspath(__file__)))
    if out.returncode != 0:
        return None
    dt = float(out.stdout.strip().splitlines()[-1])
    w = synth.WORKLOADS["c1"]
    return {"value": 2 * (w.N + w.M) / dt, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": "c1: reduced Mamba-2 layer + reduced attention layer, whole workload, one thread, %.2f s" % dt}


def cpu_baseline_attn(layer, synth, rows=48, txt_rows=4):
    """Oracle on a bounded sample: scores from a subset of text rows, attention for a subset of
    query rows of the compacted sequence; time extrapolated linearly to the whole layer."""
    import numpy as np
    import oracle
    w, t = layer.w, layer.t
    N, M, K = w.N, w.M, w.K
    f = synth.np64
    oracle.select_topk(np.zeros(4), 2)
    q_txt, k_vis = f(t["q"][N:N + txt_rows]), f(t["k"][:N])
    t0 = time.perf_counter()
    s = oracle.score_attn(q_txt, k_vis)
    t_score = (time.perf_counter() - t0) * (M / txt_rows)
    t0 = time.perf_counter()
    idx = oracle.select_topk(s, K)
    red = {k: oracle.compact(f(t[k]), idx, N, M)[0] for k in ("q", "k", "v")}
    t_sel = time.perf_counter() - t0
    Tr = K + M
    pick = np.linspace(0, Tr - 1, rows).astype(np.int32)
    t0 = time.perf_counter()
    oracle.attn(red["q"], red["k"], red["v"], rows=pick)
    t_attn = (time.perf_counter() - t0) * (Tr * (Tr + 1) / 2) / float((pick.astype(np.float64) + 1).sum())
    tot = t_score + t_sel + t_attn
    return {"value": (N + M) / tot, "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "extrapolated: scores from %d of %d text rows, attention for %d of %d query rows "
                      "(scaled by causal work); est. %.0f s for the whole layer" % (txt_rows, M, rows, Tr, tot)}


def profile_run(torch, strd, synth, name, budget, steps, warmup, dev):
    from dataclasses import replace
    wname, kind = WORKLOADS[name]
    w = replace(synth.WORKLOADS[wname], budget=budget)
    layer = (MambaLayer if kind == "mamba" else AttnLayer)(torch, strd, synth, w, dev)
    for _ in range(warmup + steps):
        layer.step()
    torch.cuda.synchronize()
    rows, row_elems = 16384, 8192                       # 16384 rows x 16 KiB = 256 MiB
    src = torch.empty(rows, row_elems, dtype=torch.bfloat16, device=dev).normal_()
    dst = torch.empty_like(src)
    ident = torch.arange(rows, dtype=torch.int32, device=dev)
    for _ in range(5):
        strd.compact(src, ident, rows, 0, out=dst)
    torch.cuda.synchronize()
    Tr = w.K + w.M
    print(json.dumps({"profile": name, "steps": warmup + steps, "mixer_kernel": layer.mixer_name,
                      "mixer_algorithmic_bytes_per_launch": layer.mixer_bytes(Tr),
                      "compact_algorithmic_bytes_per_launch": layer.compact_bytes(),
                      "calibration_copy": {"kernel": "compact_kernel", "launches": 5,
                                           "read_bytes_per_launch": rows * row_elems * 2 + rows * 4,
                                           "write_bytes_per_launch": rows * row_elems * 2}}))


def stack_model(torch, strd, synth, dev):
    """Modelled time of the mixers of the 62-layer hybrid under the paper's named schedules, from
    per-layer times measured here at every (layer kind, token count) a schedule visits."""
    from paper_2603_00198_amd.stack import model_stack_time
    w = synth.WORKLOADS["c4"]
    N0, M = w.N, w.M
    hidden = synth.hidden_states(w, dev)
    tm, ta = synth.mamba_inputs(w, hidden), synth.attn_inputs(w, hidden)
    hb = hidden.to(torch.bfloat16)
    del hidden
    sm, sa = w.mamba, w.attn
    types = strd.hybrid_layout()
    mix_cache, red_cache = {}, {}

    def rows(t, keys, n):      # the first n vision rows and the text rows of full-length tensors
        return [torch.cat([t[k][:n], t[k][N0:]]).contiguous() for k in keys]

    def mixer_time(kind, n):
        if (kind, n) not in mix_cache:
            if kind == "mamba":
                x, dt, B, C = rows(tm, ("x", "dt", "B", "C"), n)
                fn = lambda: strd.ssd_prefill(x, dt, tm["A"], B, C, chunk=sm.chunk, want_state=False)
            else:
                q, k, v = rows(ta, ("q", "k", "v"), n)
                fn = lambda: strd.attn_prefill(q, k, v)
            mix_cache[(kind, n)] = 1e-3 * time_events(torch, fn, iters=5 if kind == "attn" and n > 16384 else 10, warmup=2)
        return mix_cache[(kind, n)]

    def reduce_time(kind, n_in, k):
        if (kind, n_in, k) not in red_cache:
            if kind == "mamba":
                x, dt, B, C = rows(tm, ("x", "dt", "B", "C"), n_in)
                hid = torch.cat([hb[:n_in], hb[N0:]]).contiguous()
                Bv, Ct, dtv = B[:n_in].contiguous(), C[n_in:].contiguous(), dt[:n_in].contiguous()

                def fn():
                    idx = strd.select_topk(strd.score_mamba(Bv, Ct, dtv), k)
                    strd.compact_batch([x, B, C, dt, hid], idx, n_in, M)
            else:
                q, kk, v = rows(ta, ("q", "k", "v"), n_in)
                hid = torch.cat([hb[:n_in], hb[N0:]]).contiguous()
                qt, kv = q[n_in:].contiguous(), kk[:n_in].contiguous()

                def fn():
                    idx = strd.select_topk(strd.score_attn(qt, kv), k)
                    strd.compact_batch([q, kk, v, hid], idx, n_in, M)
            red_cache[(kind, n_in, k)] = 1e-3 * time_events(torch, fn, iters=10, warmup=2)
        return red_cache[(kind, n_in, k)]

    out = {}
    for name in strd.NAMED_SCHEDULES:
        alpha = strd.schedule_named(name)
        K = strd.schedule_budgets(alpha, N0, K_min=0)
        red, full = model_stack_time(types, K, N0, mixer_time, reduce_time)
        out[name] = {"mean_retention": sum(K) / (len(K) * N0), "mixers_full_ms": 1e3 * full, "mixers_reduced_ms": 1e3 * red,
                     "speedup": full / red}
    print(json.dumps({
        "stack_model": out, "N0": N0, "M": M, "layers": {"mamba": types.count(strd.LAYER_MAMBA),
                                                          "attn": types.count(strd.LAYER_ATTN),
                                                          "mlp_not_modelled": types.count(strd.LAYER_MLP)},
        "layer_ms": {"%s@%d" % k: 1e3 * v for k, v in sorted(mix_cache.items())},
        "note": "sum of measured per-layer times (mixer at each layer's token count + score/select/compact at the "
                "reducing layers) over the 28 Mamba-2 and 6 attention layers of the 62-layer hybrid, c4 shapes; "
                "MLP layers, projections and norms are outside this library and not in either sum",
        "context": PAPER_CONTEXT}))


def variants(torch, strd, synth, dev):
    """Average-pool reduction and the decode hand-off at the shapes of c2 / c3 (random inputs: only
    the shapes matter for these bandwidth kernels)."""
    wm, wa = synth.WORKLOADS["c2"], synth.WORKLOADS["c3"]
    out = {}
    hid = torch.randn(wm.T, wm.d_model, device=dev).to(torch.bfloat16)
    us = 1e3 * time_graph(torch, lambda: strd.avgpool(hid, wm.N, wm.M, wm.K))
    nbytes = 2 * wm.d_model * (wm.T + wm.K + wm.M)
    out["avgpool_c2_hidden"] = {"us": us, "GBps": nbytes / us * 1e-3, "frac_hbm": nbytes / us * 1e-3 / HBM_PEAK_GBS}
    m = wm.mamba
    x = torch.randn(m.H, m.P, device=dev).to(torch.bfloat16)
    B = torch.randn(m.G, m.n, device=dev).to(torch.bfloat16)
    C = torch.randn(m.G, m.n, device=dev).to(torch.bfloat16)
    dt = torch.rand(m.H, device=dev) + 0.1
    A = -torch.exp(2 * torch.rand(m.H, device=dev))
    S = torch.randn(m.H, m.P, m.n, device=dev)
    us = 1e3 * time_graph(torch, lambda: strd.ssd_decode_step(x, dt, A, B, C, None, S))
    nbytes = 8 * m.H * m.P * m.n
    out["ssd_decode_step_c2"] = {"us": us, "GBps": nbytes / us * 1e-3, "frac_hbm": nbytes / us * 1e-3 / HBM_PEAK_GBS}
    a = wa.attn
    q = torch.randn(a.Hq, a.d, device=dev).to(torch.bfloat16)
    for tag, T in (("reduced_cache", wa.K + wa.M + 1), ("full_cache", wa.T + 1)):
        kc = torch.randn(T, a.Hkv, a.d, device=dev).to(torch.bfloat16)
        vc = torch.randn(T, a.Hkv, a.d, device=dev).to(torch.bfloat16)
        ws = torch.empty(strd.lib().strd_attn_decode_step_workspace(T, a.Hq, a.Hkv, a.d, 1), dtype=torch.uint8,
                         device=dev)
        us = 1e3 * time_graph(torch, lambda: strd.attn_decode_step(q, kc, vc, ws=ws))
        nbytes = 4 * T * a.Hkv * a.d
        out["attn_decode_step_c3_" + tag] = {"T": T, "us": us, "GBps": nbytes / us * 1e-3,
                                             "frac_hbm": nbytes / us * 1e-3 / HBM_PEAK_GBS}
    # packed batch: 16 clips of 8 frames (2048 vision + 64 text tokens, 25 %) scored, selected and
    # compacted by one set of launches, against the same 16 sequences one call at a time
    nseq, nv, mt = 16, 2048, 64
    seqs = [(nv, mt, nv // 4)] * nseq
    rows = nseq * (nv + mt)
    xs = torch.randn(rows, m.H, m.P, device=dev).to(torch.bfloat16)
    Bs = (torch.randn(rows, m.G, m.n, device=dev) / m.n ** 0.5).to(torch.bfloat16)
    Cs = torch.randn(rows, m.G, m.n, device=dev).to(torch.bfloat16)
    dts = torch.rand(rows, m.H, device=dev) + 0.1
    hs = torch.randn(rows, wm.d_model, device=dev).to(torch.bfloat16)

    def packed():
        sc = strd.score_mamba_varlen(Bs, Cs, dts, seqs)
        ix = strd.select_topk_varlen(sc, seqs)
        strd.compact_varlen([xs, Bs, Cs, dts, hs], ix, seqs)

    def one_by_one():
        for b in range(nseq):
            r0 = b * (nv + mt)
            sc = strd.score_mamba(Bs[r0:r0 + nv], Cs[r0 + nv:r0 + nv + mt], dts[r0:r0 + nv])
            ix = strd.select_topk(sc, nv // 4)
            strd.compact_batch([t[r0:r0 + nv + mt] for t in (xs, Bs, Cs, dts, hs)], ix, nv, mt)

    us_p, us_1 = 1e3 * time_events(torch, packed, iters=10), 1e3 * time_events(torch, one_by_one, iters=10)
    out["reduce_16_clips_of_2048"] = {"packed_us": us_p, "one_call_per_sequence_us": us_1, "gain": us_1 / us_p,
                                      "input_tokens_per_s_packed": rows / (us_p * 1e-6)}
    # the in-projection of a Mamba-2 block at c4 (33 024 tokens, 4096 -> 18 560): the library product and
    # the kernel of this library that needs no handle
    w4 = synth.WORKLOADS["c4"]
    nd = 2 * w4.mamba.H * w4.mamba.P + 2 * w4.mamba.G * w4.mamba.n + w4.mamba.H
    u = torch.randn(w4.T, w4.d_model, device=dev).to(torch.bfloat16)
    wp = (torch.randn(w4.d_model, nd, device=dev) / w4.d_model ** 0.5).to(torch.bfloat16)
    po = torch.empty(w4.T, nd, dtype=torch.bfloat16, device=dev)
    flops = 2.0 * w4.T * w4.d_model * nd
    ms_lib = time_events(torch, lambda: strd.linear_library(u, wp, out=po), iters=5)
    ms_own = time_events(torch, lambda: strd.linear_mfma(u, wp, out=po), iters=5)
    out["in_projection_c4"] = {"T": w4.T, "Kd": w4.d_model, "Nd": nd, "library_ms": ms_lib, "own_kernel_ms": ms_own,
                               "library_TFLOPs": flops / ms_lib * 1e-9, "own_kernel_TFLOPs": flops / ms_own * 1e-9,
                               "own_kernel_frac_of_bf16_peak": flops / ms_own * 1e-9 / MFMA_BF16_PEAK_TFLOPS}
    del u, wp, po
    out["note"] = ("average-pool baseline of the reduction-type ablation on the residual stream; one decode token from "
                   "the state / the key-value rows a prefill leaves (25% budget vs none); device time per call from a "
                   "graph of 20 calls; score + select + compact of a packed batch of short sequences (one set of "
                   "launches) against one call per sequence, event-timed; not part of the timed step")
    return out


def batch_mode(torch, strd, synth, name, budget, batch, steps, warmup, dev):
    """`batch` independent sequences of the workload, one stream each (every entry point takes one
    sequence; a batch is a set of streams): the steps of different sequences overlap on the GPU, which
    is what the latency-bound parts of a step (top-k, launches, the scan's serial chain) leave room
    for.  Reports the aggregate rate beside the single-sequence one."""
    import dataclasses
    w0 = dataclasses.replace(synth.WORKLOADS[name], budget=budget)
    cls = MambaLayer if w0.mamba is not None and name != "c3" else AttnLayer
    layers = [cls(torch, strd, synth, dataclasses.replace(w0, seed=w0.seed + 17 * i), dev) for i in range(batch)]
    streams = [torch.cuda.Stream() for _ in range(batch)]

    def round_all():
        for layer, st in zip(layers, streams):
            with torch.cuda.stream(st):
                layer.step()

    def timed(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    for _ in range(warmup):
        round_all()
        layers[0].step()
    ms_one = timed(layers[0].step, steps)
    ms_round = timed(round_all, steps)
    print(json.dumps({
        "batch": batch, "workload": name, "layer": layers[0].kind, "ms_per_step_single_sequence": ms_one,
        "ms_per_round_of_batch": ms_round, "tokens_per_s_single": w0.T / (ms_one * 1e-3),
        "tokens_per_s_batch": batch * w0.T / (ms_round * 1e-3), "gain": batch * ms_one / ms_round,
        "note": "one stream per sequence, default priorities; inputs resident; same six calls per sequence"}))


def block_stack(torch, strd, synth, dev, iters=5):
    """Hidden-to-hidden 8-block stack (c4): full against progressively reduced, event-timed."""
    from paper_2603_00198_amd import blocks
    w = synth.WORKLOADS["c4"]
    kinds = synth.C4_LAYERS
    wts = [synth.mamba_block_weights(w, dev, l) if k == "mamba" else synth.attn_block_weights(w, dev, l)
           for l, k in enumerate(kinds)]
    hidden = synth.hidden_states(w, dev).to(torch.bfloat16)
    budgets = strd.schedule_budgets(list(synth.C4_RETAIN), w.N)
    full = [w.N] * len(kinds)
    run = lambda b: blocks.run_blocks(kinds, wts, hidden, w.N, w.M, b, w.mamba, w.attn)
    out = {}
    for name, b in (("full", full), ("reduced", budgets)):
        ms = time_events(torch, lambda: run(b), iters=iters, warmup=2)
        out[name] = {"ms": ms, "input_tokens_per_s": w.T / (ms * 1e-3)}
    # where the time of one full Mamba-2 block goes
    h1 = hidden
    parts = {}
    s, wt = w.mamba, wts[0]
    u = strd.rmsnorm(h1, wt["norm_w"])
    parts["rmsnorm_us"] = 1e3 * time_events(torch, lambda: strd.rmsnorm(h1, wt["norm_w"]), iters=iters)
    parts["in_proj_us"] = 1e3 * time_events(torch, lambda: (strd.linear(u, wt["W_z"]), strd.linear(u, wt["W_xbcdt"])), iters=iters)
    xbcdt = strd.linear(u, wt["W_xbcdt"])
    z = strd.linear(u, wt["W_z"])
    d_inner, gn = s.H * s.P, s.G * s.n
    parts["conv1d_silu_us"] = 1e3 * time_events(
        torch, lambda: strd.conv1d_silu(xbcdt, wt["conv_w"], wt["conv_b"], d_inner, gn), iters=iters)
    parts["softplus_dt_us"] = 1e3 * time_events(
        torch, lambda: strd.softplus_dt(xbcdt[:, d_inner + 2 * gn:], wt["dt_bias"]), iters=iters)
    x, B, C = strd.conv1d_silu(xbcdt, wt["conv_w"], wt["conv_b"], d_inner, gn)
    dt = strd.softplus_dt(xbcdt[:, d_inner + 2 * gn:], wt["dt_bias"])
    x3, B3, C3 = x.view(w.T, s.H, s.P), B.view(w.T, s.G, s.n), C.view(w.T, s.G, s.n)
    parts["ssd_prefill_us"] = 1e3 * time_events(
        torch, lambda: strd.ssd_prefill(x3, dt, wt["A"], B3, C3, wt["D"], chunk=s.chunk, want_state=False), iters=iters)
    y, _ = strd.ssd_prefill(x3, dt, wt["A"], B3, C3, wt["D"], chunk=s.chunk, want_state=False)
    y2 = y.view(w.T, d_inner)
    parts["gated_rmsnorm_us"] = 1e3 * time_events(torch, lambda: strd.gated_rmsnorm(y2, z, wt["gnorm_w"], s.G), iters=iters)
    g = strd.gated_rmsnorm(y2, z, wt["gnorm_w"], s.G)
    parts["out_proj_us"] = 1e3 * time_events(torch, lambda: strd.linear(g, wt["W_out"], residual=h1), iters=iters)
    parts["in_proj_rocblas_us"] = 1e3 * time_events(
        torch, lambda: (strd.linear_library(u, wt["W_z"]), strd.linear_library(u, wt["W_xbcdt"])), iters=iters)
    parts["out_proj_rocblas_us"] = 1e3 * time_events(torch, lambda: strd.linear_library(g, wt["W_out"], residual=h1), iters=iters)
    eb = 2
    glue_bytes = {"rmsnorm": 2 * w.T * w.d_model * eb, "conv1d_silu": 2 * w.T * (d_inner + 2 * gn) * eb,
                  "gated_rmsnorm": 3 * w.T * d_inner * eb}
    parts["glue_GBps"] = {k: v / (parts[k + "_us"] * 1e-6) / 1e9 for k, v in glue_bytes.items()}
    print(json.dumps({
        "block_stack": out, "speedup": out["full"]["ms"] / out["reduced"]["ms"], "workload": "c4: %s, N=%d M=%d, d_model=%d"
        % ("+".join(kinds), w.N, w.M, w.d_model), "budgets": budgets, "full_mamba_block_parts": parts,
        "note": "hidden-to-hidden: pre-norm, projections (own kernel from one 256x256 tile per CU up, rocBLAS below; the same two projections by rocBLAS alone beside them), conv1d+SiLU, softplus, score/select/compact at the "
                "reducing blocks, mixer, gated norm, out-projection + residual; no MLP blocks"}))


def matrix_core_rate(torch, strd, dev):
    """TFLOP/s of back-to-back bf16 32x32x16 products on register-resident operands (no loads, no LDS),
    with constant and with random operands: what the matrix cores of THIS chip sustain at the clock
    its power management allows, beside the published 2.5 PFLOP/s the roofline fractions are taken of."""
    out = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    res = {}
    for tag, rnd, small in (("constant_operands", 0, False), ("random_operands", 1, False),
                            ("random_operands_16x16x32", 1, True)):
        strd.mfma_rate_probe(512, 2000, rnd, out, small_products=small)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        strd.mfma_rate_probe(512, 10000, rnd, out, small_products=small)
        e1.record()
        torch.cuda.synchronize()
        res[tag + "_TFLOPs"] = 512 * 4 * 10000 * 32 * 32768 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    res["note"] = ("strd_mfma_rate_probe: 2 waves per SIMD issuing only products; real activations look like the random "
                   "case to the multipliers, and the clock under full-rate products follows the power they draw")
    return res


def median(vals):
    v = sorted(vals)
    n = len(v)
    return 0.0 if n == 0 else (v[n // 2] if n % 2 else 0.5 * (v[n // 2 - 1] + v[n // 2]))


def measure(torch, strd, synth, name, budget, steps, warmup, dev):
    from dataclasses import replace
    wname, kind = WORKLOADS[name]
    w = replace(synth.WORKLOADS[wname], budget=budget)
    layer = (MambaLayer if kind == "mamba" else AttnLayer)(torch, strd, synth, w, dev)
    # whole reduced step, with the mixer bracketed by its own event pair inside the timed region
    for _ in range(warmup):
        layer.step()
    torch.cuda.synchronize()
    layer.mixer_ev = EventPairs(torch)
    t0 = time.perf_counter()
    for _ in range(steps):
        layer.step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps
    ms_mixer = layer.mixer_ev.mean_ms()
    ms_mixer_median = median([a.elapsed_time(b) for a, b in layer.mixer_ev.pairs])
    layer.mixer_ev = None
    # the same K steps again, each bracketed by its own event pair: the median step
    step_ev = EventPairs(torch)
    for _ in range(steps):
        step_ev.wrap(layer.step)
    torch.cuda.synchronize()
    ms_step_median = median([a.elapsed_time(b) for a, b in step_ev.pairs])
    # the same step captured once into a HIP graph and replayed (no per-launch host work)
    ms_graph = None
    try:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            layer.step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                layer.step()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t0) * 1e3 / steps
    except Exception as exc:  # graph capture is an extra figure, never the headline
        print("bench.py: graph replay skipped: %s" % exc, file=sys.stderr)
    calls = {
        "score_us": 1e3 * time_events(torch, layer.score),
        "select_topk_us": 1e3 * time_events(torch, layer.select),
        "compact_us": 1e3 * time_events(torch, layer.compact),
        "mixer_reduced_us": 1e3 * ms_mixer,
        "mixer_reduced_median_us": 1e3 * ms_mixer_median,
    }
    # The event pair around a single short call also sees the host's launch path (the queue is
    # empty when it starts); a graph of 20 back-to-back calls gives the device time per call.
    dev_calls = {}
    try:
        dev_calls = {"score_us": 1e3 * time_graph(torch, layer.score),
                     "select_topk_us": 1e3 * time_graph(torch, layer.select),
                     "compact_us": 1e3 * time_graph(torch, layer.compact)}
    except Exception as exc:
        print("bench.py: per-call graph timing skipped: %s" % exc, file=sys.stderr)
    full_iters = max(3, min(20, int(200.0 / max(ms_mixer * (w.T / (w.K + w.M)), 1e-3))))
    ms_full = time_events(torch, layer.mixer_full, iters=full_iters, warmup=2)
    calls["mixer_full_us"] = 1e3 * ms_full
    Tr = w.K + w.M
    sel_compact_gbs = (layer.compact_bytes() + 4 * w.N) / ((calls["select_topk_us"] + calls["compact_us"]) * 1e-6) / 1e9
    sel_compact_dev = None
    if dev_calls:
        sel_compact_dev = (layer.compact_bytes() + 4 * w.N) / ((dev_calls["select_topk_us"] + dev_calls["compact_us"]) * 1e-6) / 1e9
    traffic = measured_traffic(name, budget, layer.mixer_name)
    if layer.mixer_bound == "hbm":
        ach = layer.mixer_bytes(Tr) / (ms_mixer * 1e-3) / 1e9
        tf_step = layer.mixer_flops(Tr, KERNEL_STEP) / (ms_mixer * 1e-3) / 1e12
        tf_chunk = layer.mixer_flops(Tr, layer.s.chunk) / (ms_mixer * 1e-3) / 1e12
        roof = {"bound": "hbm", "kernel": layer.mixer_name, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": traffic,
                "mfma_tflops": tf_step, "mfma_frac": tf_step / MFMA_BF16_PEAK_TFLOPS,
                "mfma_tflops_at_chunk_%d" % layer.s.chunk: tf_chunk,
                "mfma_frac_at_chunk_%d" % layer.s.chunk: tf_chunk / MFMA_BF16_PEAK_TFLOPS,
                "mfma_note": "causal flop count of the chunked scan at the kernel's own step of %d tokens (what it has to "
                             "execute); beside it the count of the same scan at the workload's chunk of %d, which this "
                             "kernel never executes" % (KERNEL_STEP, layer.s.chunk)}
    else:
        ach = layer.mixer_flops(Tr) / (ms_mixer * 1e-3) / 1e12
        roof = {"bound": "mfma", "kernel": layer.mixer_name, "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic}
    # every call against both published peaks (algorithmic work / event-timed duration)
    def fr(nbytes, flops, us):
        return {"us": us, "GBps": nbytes / (us * 1e-6) / 1e9, "frac_hbm": nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "TFLOPs": flops / (us * 1e-6) / 1e12, "frac_mfma": flops / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    sb, sf = layer.score_work()
    per_call = {
        "score": fr(sb, sf, dev_calls.get("score_us", calls["score_us"])),
        "select_topk": fr(4 * w.N + 4 * w.K, 0.0, dev_calls.get("select_topk_us", calls["select_topk_us"])),
        "compact": fr(layer.compact_bytes(), 0.0, dev_calls.get("compact_us", calls["compact_us"])),
        "mixer_reduced": fr(layer.mixer_bytes(Tr), layer.mixer_flops(Tr), calls["mixer_reduced_us"]),
        "mixer_full": fr(layer.mixer_bytes(w.T), layer.mixer_flops(w.T), calls["mixer_full_us"]),
        "note": "algorithmic bytes and flops of each call over its duration (score, select_topk, compact: device time "
                "per call from a graph of 20 calls; mixers: HIP events on the stream)",
    }
    fused = None
    if kind == "mamba":   # variant: the scan gathers its inputs itself (same y, bit for bit; see tests)
        layer.fused = True
        for _ in range(warmup):
            layer.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            layer.step()
        torch.cuda.synchronize()
        ms_fused = (time.perf_counter() - t0) * 1e3 / steps
        fused = {"ms_per_step": ms_fused, "tokens_per_s": w.T / (ms_fused * 1e-3), "speedup_vs_full": ms_full / ms_fused,
                 "compact_us": 1e3 * time_events(torch, layer.compact),
                 "mixer_reduced_us": 1e3 * time_events(torch, layer.mixer_reduced),
                 "note": "ssd_prefill_gather reads x, dt, B, C through idx; only the residual stream is compacted"}
        layer.fused = False
        fused["score_mamba_full_us"] = 1e3 * time_events(torch, layer.score_full)
    s = w.mamba if kind == "mamba" else w.attn
    res = {
        "layer": kind, "workload": name,
        "config": "%s: single %s layer, %d vision + %d text tokens, budget %.0f%% (K=%d), batch 1, %s"
                  % (name, "Mamba-2" if kind == "mamba" else "attention", w.N, w.M, 100 * budget, w.K, repr(s)),
        "N": w.N, "M": w.M, "K": w.K, "budget": budget, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_step, "ms_per_step_median": ms_step_median, "graph_replay_ms_per_step": ms_graph,
        "tokens_per_s": w.T / (ms_step * 1e-3),
        "retained_tokens_per_s": Tr / (ms_step * 1e-3), "speedup_vs_full": ms_full / ms_step,
        "calls": calls, "calls_device_us": dev_calls, "select_plus_compact_GBps": sel_compact_gbs,
        "select_plus_compact_device_GBps": sel_compact_dev,
        "select_plus_compact_device_frac_of_hbm": None if sel_compact_dev is None else sel_compact_dev / HBM_PEAK_GBS,
        "select_plus_compact_frac_of_hbm": sel_compact_gbs / HBM_PEAK_GBS, "roofline": roof,
        "per_call_roofline": per_call,
    }
    if fused:
        res["gather_fused_variant"] = fused
    return res, layer


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path uses no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2603_00198_amd as strd
    from paper_2603_00198_amd import synth
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    name = args.workload
    if args.stack_model:
        stack_model(torch, strd, synth, dev)
        return
    if args.block_stack:
        block_stack(torch, strd, synth, dev)
        return
    if args.variants:
        print(json.dumps({"variants": variants(torch, strd, synth, dev)}))
        return
    if args.batch > 0:
        batch_mode(torch, strd, synth, name, args.budget, args.batch, args.steps, args.warmup, dev)
        return
    if args.profile:
        profile_run(torch, strd, synth, name, args.budget, args.steps, args.warmup, dev)
        return
    res, layer = measure(torch, strd, synth, name, args.budget, args.steps, args.warmup, dev)
    w = layer.w
    line = {
        "metric": "retained-token prefill tokens/s per layer at 25% budget; speedup vs full prefill",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "ms_per_step_median": res["ms_per_step_median"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": res["config"],
                   "tokens_counted": "input tokens N+M per reduced-layer step (score+select+compact+mixer)",
                   "timing": "value = (N+M) / wall-clock mean of the K timed steps; ms_per_step_median = median of the "
                             "same K steps timed one by one with HIP events",
                   "parallelism": "1 GPU"},
        "speedup_vs_full": res["speedup_vs_full"], "retained_tokens_per_s": res["retained_tokens_per_s"],
        "graph_replay_ms_per_step": res["graph_replay_ms_per_step"],
        "calls_us": res["calls"], "calls_device_us": res["calls_device_us"],
        "select_plus_compact_device_GBps": res["select_plus_compact_device_GBps"],
        "select_plus_compact_device_frac_of_hbm": res["select_plus_compact_device_frac_of_hbm"],
        "select_plus_compact_GBps": res["select_plus_compact_GBps"],
        "select_plus_compact_frac_of_hbm": res["select_plus_compact_frac_of_hbm"],
        "roofline": res["roofline"], "per_call_roofline": res["per_call_roofline"], "context": PAPER_CONTEXT,
    }
    if "gather_fused_variant" in res:
        line["gather_fused_variant"] = res["gather_fused_variant"]
        line["next_rows"] = {"score_mamba_full_us": line["gather_fused_variant"].pop("score_mamba_full_us"),
                             "note": "Full Mamba Dynamic score (decayed |w_tj|) on the same inputs; an ablation "
                                     "row, not part of the timed step"}
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline_mamba(layer, synth) if layer.kind == "mamba" \
            else cpu_baseline_attn(layer, synth)
    del layer
    torch.cuda.empty_cache()
    extras = not args.no_extras and name == "c5m"
    if extras:
        # the attention layer of the same long-video configuration, with the same steps and warm-up,
        # then the two smaller single-layer workloads
        ares, alayer = measure(torch, strd, synth, "c5a", args.budget, args.steps, args.warmup, dev)
        if not args.no_cpu_baseline:
            ares["cpu_baseline"] = cpu_baseline_attn(alayer, synth)
        line["attention_layer"] = ares
        del alayer
        torch.cuda.empty_cache()
        line["other_workloads"] = {}
        for other in ("c2", "c3"):
            ores, olayer = measure(torch, strd, synth, other, args.budget, args.steps, args.warmup, dev)
            ores.pop("per_call_roofline", None)
            if "gather_fused_variant" in ores:
                ores["gather_fused_variant"].pop("score_mamba_full_us", None)
            line["other_workloads"][other] = ores
            del olayer
            torch.cuda.empty_cache()
        line.setdefault("next_rows", {})["variants"] = variants(torch, strd, synth, dev)
        line["matrix_core_rate_probe"] = matrix_core_rate(torch, strd, dev)
    if not args.no_cpu_baseline:
        line["cpu_baseline"]["single_thread_c1"] = cpu_single_thread_c1(torch, synth)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
