"""Element-by-element parity of the HIP library (through the C ABI) with the CPU fp64 oracle on
identical seeded inputs, at sizes the oracle finishes in seconds that still span several tiles
and a ragged tail.  Needs a GPU: run with -m gpu."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_00198_amd as strd
from paper_2603_00198_amd import synth
from util import TOL, assert_close, assert_topk_equivalent

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print("[case] " + msg, flush=True)


# ------------------------------------------------------------------ compact ----------------
@pytest.mark.parametrize("N,M,K,row_elems,dtype", [
    (1024, 32, 512, 256, torch.float32),      # tiny pair, hidden rows
    (1000, 7, 333, 130, torch.bfloat16),      # 260-byte rows: not a multiple of 16
    (4096, 128, 1024, 4096, torch.bfloat16),  # 8 KB rows
    (300, 0, 300, 2, torch.float32),          # K = N, no text
    (300, 5, 0, 8, torch.float32),            # nothing retained
    (77, 3, 20, 1, torch.float32),            # 4-byte rows (dt of one head)
])
def test_compact_bit_exact(N, M, K, row_elems, dtype):
    _say("compact N=%d M=%d K=%d row=%d %s" % (N, M, K, row_elems, dtype))
    g = torch.Generator().manual_seed(N + K)
    src = torch.randn(N + M, row_elems, generator=g).to(dtype)
    idx = torch.sort(torch.randperm(N, generator=g)[:K]).values.to(torch.int32)
    pos_in = torch.randperm(10 * (N + M), generator=g)[: N + M].to(torch.int32)
    dst, pos = strd.compact(src.to(DEV), idx.to(DEV), N, M, pos_in=pos_in.to(DEV))
    raw = src.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).numpy()
    want, want_pos = oracle.compact(raw, idx.numpy(), N, M, pos_in=pos_in.numpy())
    got = dst.cpu().view(torch.int16 if dtype == torch.bfloat16 else torch.int32).numpy()
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(pos.cpu().numpy(), want_pos)
    _, pos_id = strd.compact(None, idx.to(DEV), N, M, want_pos=True)
    np.testing.assert_array_equal(pos_id.cpu().numpy(), oracle.compact(raw, idx.numpy(), N, M)[1])


def test_compact_batch_bit_exact():
    _say("compact_batch 5 tensors + positions")
    N, M, K = 3000, 70, 811
    g = torch.Generator().manual_seed(1)
    shapes = [((64, 32), torch.bfloat16), ((8, 16), torch.bfloat16), ((24,), torch.float32), ((130,), torch.bfloat16),
              ((4096,), torch.bfloat16)]
    srcs = [torch.randn((N + M,) + shp, generator=g).to(dt) for shp, dt in shapes]
    idx = torch.sort(torch.randperm(N, generator=g)[:K]).values.to(torch.int32)
    pos_in = torch.randperm(5 * (N + M), generator=g)[: N + M].to(torch.int32)
    outs, pos = strd.compact_batch([t.to(DEV) for t in srcs], idx.to(DEV), N, M, pos_in=pos_in.to(DEV))
    for t, o in zip(srcs, outs):
        raw = t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).numpy()
        want, want_pos = oracle.compact(raw, idx.numpy(), N, M, pos_in=pos_in.numpy())
        got = o.cpu().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).numpy()
        np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(pos.cpu().numpy(), want_pos)


# ------------------------------------------------------------------ select_topk ------------
def _topk_case(scores, K):
    got = strd.select_topk(torch.from_numpy(scores).to(DEV), K).cpu().numpy()
    want = oracle.select_topk(scores.astype(np.float64), K)
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("N,K", [(1, 1), (5, 3), (1024, 512), (4097, 1000), (8192, 2048), (10000, 9999),
                                 (50000, 1), (131072, 32768), (131072, 13107), (200003, 65536)])
def test_select_topk_bit_exact_random(N, K):
    _say("topk random N=%d K=%d" % (N, K))
    r = np.random.default_rng(N * 7 + K)
    _topk_case(r.random(N, dtype=np.float32) ** 4, K)


@pytest.mark.parametrize("levels", [1, 2, 7, 300])
def test_select_topk_ties_go_to_lowest_index(levels):
    _say("topk ties levels=%d" % levels)
    r = np.random.default_rng(levels)
    N = 20000
    s = (r.integers(0, levels, N) / np.float32(levels)).astype(np.float32)
    s[::97] = -0.0 if levels > 1 else s[::97]
    for K in (1, 777, N // 2, N - 1, N):
        _topk_case(s, K)


@pytest.mark.parametrize("in_bin", [1, 2, 63, 64, 65, 200])
@pytest.mark.parametrize("N", [6000, 30000])
def test_select_topk_small_last_bin(N, in_bin):
    """Scores built from their bit patterns so that the first 11-bit digit of key - min(key) leaves
    exactly `in_bin` candidates, some of them equal: at most 64 are ranked directly by one wave, more
    go through another digit.  The K-th score is placed on every rank inside that bin."""
    _say("topk small last bin N=%d in_bin=%d" % (N, in_bin))
    r = np.random.default_rng(N + in_bin)
    top = r.integers(0, 2048, N)                      # first digit of the 22-bit offset
    top[top == 1000] = 999
    off = (top.astype(np.int64) << 11) + r.integers(0, 2048, N)
    off[0], off[1] = 0, (1 << 22) - 1                 # the offsets span exactly 22 bits
    where = r.choice(np.arange(2, N), in_bin, replace=False)
    low = r.integers(0, 2048, in_bin)
    low[: in_bin // 3] = low[-1]                      # duplicates of one candidate
    off[where] = (1000 << 11) + low
    s = (np.uint32(0x3F800000) + off.astype(np.uint32)).view(np.float32)   # positive floats, order = offset order
    above = int((off >= (1001 << 11)).sum())
    for rank in sorted({1, 2, in_bin // 3, in_bin // 2, in_bin - 1, in_bin} - {0}):
        _topk_case(s, above + rank)


def test_select_topk_tiny_and_denormal_scores():
    _say("topk denormals")
    r = np.random.default_rng(3)
    s = (r.random(9000, dtype=np.float32) * np.float32(1e-41)).astype(np.float32)  # denormal range
    s[100:200] = 0.0
    _topk_case(s, 4000)
    _topk_case(s, 8950)


@pytest.mark.parametrize("N,K", [(8192, 2048), (32768, 8192), (40000, 39000)])
def test_select_topk_narrow_range_and_signed_scores(N, K):
    _say("topk narrow / signed N=%d K=%d" % (N, K))
    r = np.random.default_rng(N + K)
    _topk_case(((1.0 + r.random(N)) / N).astype(np.float32), K)       # within a factor of two: two 11-bit digits
    _topk_case((1.0 + 1e-6 * r.random(N)).astype(np.float32), K)      # a few distinct values around 1: one digit
    s = r.standard_normal(N).astype(np.float32)                       # both signs: three digits
    s[::1001] = np.float32(np.inf)
    s[5::1003] = np.float32(-np.inf)
    _topk_case(s, K)


@pytest.mark.parametrize("N", [32769, 70000, 1 << 20, (1 << 20) + 1])
def test_select_topk_many_workgroup_form(N):
    """Above 32768 scores the selection runs as a chain of launches with one workgroup per 4096
    scores (up to 2^20 scores; beyond that one streaming workgroup again): a single score in the
    last tile, ties that span tiles, all scores equal, K = 1 and K = N."""
    _say("topk wide form N=%d" % N)
    r = np.random.default_rng(N)
    s = (r.random(N, dtype=np.float32) ** 3).astype(np.float32)
    for K in (1, N // 4, N - 1, N):
        _topk_case(s, K)
    t = (r.integers(0, 5, N) / np.float32(5)).astype(np.float32)      # five levels: every tile full of ties
    for K in (N // 10, N // 2 + 1):
        _topk_case(t, K)
    _topk_case(np.full(N, 0.25, dtype=np.float32), N // 3)            # all equal: the first N // 3 indices


# ------------------------------------------------------------------ scores -----------------
def _mamba_case(w, seed=0):
    h = synth.hidden_states(w, DEV, seed)
    return synth.mamba_inputs(w, h, seed)


def _attn_case(w, seed=0):
    h = synth.hidden_states(w, DEV, seed)
    return synth.attn_inputs(w, h, seed)


MAMBA_CASES = {
    "c1": synth.WORKLOADS["c1"],
    "c2-short": synth.shrink(synth.WORKLOADS["c2"], N=1500, M=37, d_model=512),
    "odd": synth.shrink(synth.WORKLOADS["c2"], N=700, M=5, d_model=128,
                        mamba=synth.MambaShape(H=6, P=24, n=40, G=3, chunk=64)),
    "n64": synth.shrink(synth.WORKLOADS["c2"], N=700, M=5, d_model=128,
                        mamba=synth.MambaShape(H=6, P=96, n=64, G=2, chunk=128)),
}
ATTN_CASES = {
    "c1": synth.WORKLOADS["c1"],
    "c3-short": synth.shrink(synth.WORKLOADS["c3"], N=1500, M=37, d_model=512),
    "odd": synth.shrink(synth.WORKLOADS["c3"], N=333, M=3, d_model=128, attn=synth.AttnShape(Hq=6, Hkv=3, d=40)),
    "d64": synth.shrink(synth.WORKLOADS["c3"], N=700, M=5, d_model=128, attn=synth.AttnShape(Hq=6, Hkv=2, d=64)),
    "c3-mid": synth.shrink(synth.WORKLOADS["c3"], N=5000, M=100, d_model=256),
}


@pytest.mark.parametrize("name", list(MAMBA_CASES))
def test_score_mamba_parity(name):
    w = MAMBA_CASES[name]
    _say("score_mamba %s N=%d M=%d %s" % (name, w.N, w.M, w.dtype))
    t = _mamba_case(w)
    N = w.N
    got = strd.score_mamba(t["B"][:N].contiguous(), t["C"][N:].contiguous(), t["dt"][:N].contiguous())
    want = oracle.score_mamba(synth.np64(t["B"][:N]), synth.np64(t["C"][N:]), synth.np64(t["dt"][:N]))
    assert_close(got.cpu().numpy(), want, TOL[synth.torch_dtype(w.dtype)], "score_mamba " + name, units=(0,))
    K = max(1, w.K)
    idx = strd.select_topk(got, K).cpu().numpy()
    assert_topk_equivalent(idx, want, K, TOL[synth.torch_dtype(w.dtype)])


FULL_CASES = {
    "c1": synth.WORKLOADS["c1"],                                                     # fp32, SIMT path
    "n64": MAMBA_CASES["n64"],                                                       # 3 heads per group (padded k)
    "odd": MAMBA_CASES["odd"],                                                       # bf16, SIMT path
    "c2-tiny": synth.shrink(synth.WORKLOADS["c2"], N=600, M=20, d_model=256),        # 16 heads per group
    "c2-ragged": synth.shrink(synth.WORKLOADS["c2"], N=300, M=37, d_model=256),      # ragged text tile
}


@pytest.mark.parametrize("a_scale", [1.0, 0.003])   # 0.003: the decay is mild over the whole sequence, every
@pytest.mark.parametrize("name", list(FULL_CASES))  # block of the suffix sum matters, not only the last tokens
def test_score_mamba_full_parity(name, a_scale):
    w = FULL_CASES[name]
    _say("score_mamba_full %s N=%d M=%d %s A x %g" % (name, w.N, w.M, w.dtype, a_scale))
    t = _mamba_case(w, seed=3)
    N = w.N
    A = (t["A"] * a_scale).contiguous()
    got = strd.score_mamba_full(t["B"][:N].contiguous(), t["C"][N:].contiguous(), t["dt"], A)
    want = oracle.score_mamba_full(synth.np64(t["B"]), synth.np64(t["C"]), synth.np64(t["dt"]), synth.np64(A), N)
    tol = TOL[synth.torch_dtype(w.dtype)]
    assert_close(got.cpu().numpy(), want, tol, "score_mamba_full " + name, units=(0,))
    K = max(1, w.K)
    assert_topk_equivalent(strd.select_topk(got, K).cpu().numpy(), want, K, tol, floor=1e-30 * want.max())


def test_score_mamba_full_without_decay_is_the_decay_free_score():
    w = FULL_CASES["c2-tiny"]
    t = _mamba_case(w, seed=4)
    N = w.N
    Bv, Ct = t["B"][:N].contiguous(), t["C"][N:].contiguous()
    full = strd.score_mamba_full(Bv, Ct, t["dt"], torch.zeros_like(t["A"]))
    free = strd.score_mamba(Bv, Ct, t["dt"][:N].contiguous())
    assert_close(full.cpu().numpy(), free.cpu().numpy().astype(np.float64), 1e-4, "A = 0")


@pytest.mark.parametrize("name", list(ATTN_CASES))
def test_score_attn_parity(name):
    w = ATTN_CASES[name]
    _say("score_attn %s N=%d M=%d %s" % (name, w.N, w.M, w.dtype))
    t = _attn_case(w)
    N = w.N
    got = strd.score_attn(t["q"][N:].contiguous(), t["k"][:N].contiguous())
    want = oracle.score_attn(synth.np64(t["q"][N:]), synth.np64(t["k"][:N]))
    tol = TOL[synth.torch_dtype(w.dtype)]
    assert_close(got.cpu().numpy(), want, tol, "score_attn " + name, units=(0,))
    assert abs(float(got.double().sum()) - 1.0) < tol
    K = max(1, w.K)
    idx = strd.select_topk(got, K).cpu().numpy()
    assert_topk_equivalent(idx, want, K, tol)


# ------------------------------------------------------------------ mixers -----------------
@pytest.mark.parametrize("name,T,extras", [("c1", 1056, False), ("c1", 544, True), ("c2-short", 300, True),
                                           ("c2-short", 1537, False), ("odd", 130, True), ("c1", 1, True),
                                           ("c1", 0, False), ("c2-short", 64, True), ("c2-short", 65, False),
                                           ("c2-short", 1, True), ("c2-short", 0, True), ("n64", 200, True),
                                           ("n64", 705, False)])
def test_ssd_prefill_parity(name, T, extras):
    w = MAMBA_CASES[name]
    s = w.mamba
    _say("ssd_prefill %s T=%d extras=%s %s" % (name, T, extras, w.dtype))
    t = _mamba_case(w, seed=T)
    x, dt, B, C = (t[k][:T].contiguous() for k in ("x", "dt", "B", "C"))
    g = torch.Generator(device=DEV).manual_seed(5)
    D = torch.randn(s.H, generator=g, device=DEV) if extras else None
    S_in = torch.randn(s.H, s.P, s.n, generator=g, device=DEV) if extras else None
    y, S_out = strd.ssd_prefill(x, dt, t["A"], B, C, D, S_in, chunk=s.chunk)
    yw, Sw = oracle.ssd_seq(synth.np64(x), synth.np64(dt), synth.np64(t["A"]), synth.np64(B), synth.np64(C),
                            None if D is None else synth.np64(D), None if S_in is None else synth.np64(S_in))
    tol = TOL[synth.torch_dtype(w.dtype)]
    assert_close(synth.np64(y), yw, tol, "ssd y", units=(1,))
    assert_close(synth.np64(S_out), Sw, tol, "ssd S_out", units=(0,))


@pytest.mark.parametrize("T", [2, 63, 64, 65, 128, 129, 191, 192, 193, 256, 257, 320, 449, 512, 513])
def test_ssd_prefill_step_boundaries(T):
    """Sequence lengths around the 64-token steps and around the look-ahead of the copies (one to
    nine steps): dense with D and a carried-in state, and through an index list."""
    _say("ssd_prefill step boundaries T=%d" % T)
    H, P, G, n = 4, 64, 2, 128
    g = torch.Generator().manual_seed(1000 + T)
    M = min(7, T - 1)
    K = T - M
    N = 2 * K + 3
    rows = N + M
    x = torch.randn(rows, H, P, generator=g).to(torch.bfloat16)
    B = (torch.randn(rows, G, n, generator=g) / n ** 0.5).to(torch.bfloat16)
    C = torch.randn(rows, G, n, generator=g).to(torch.bfloat16)
    dt = torch.nn.functional.softplus(torch.randn(rows, H, generator=g))
    A = -torch.exp(2 * torch.rand(H, generator=g))
    D = torch.randn(H, generator=g)
    S_in = torch.randn(H, P, n, generator=g)
    idx = torch.sort(torch.randperm(N, generator=g)[:K]).values.to(torch.int32)
    keep = torch.cat([idx.long(), torch.arange(N, rows)])
    f = synth.np64
    y_ref, S_ref = oracle.ssd_seq(f(x[keep]), f(dt[keep]), f(A), f(B[keep]), f(C[keep]), f(D), f(S_in))
    dev = lambda t: t.to(DEV)
    y, S = strd.ssd_prefill(dev(x[keep].contiguous()), dev(dt[keep].contiguous()), dev(A), dev(B[keep].contiguous()),
                            dev(C[keep].contiguous()), D=dev(D), S_in=dev(S_in))
    assert_close(f(y), y_ref, TOL[torch.bfloat16], "y", units=(1,))
    assert_close(f(S), S_ref, TOL[torch.bfloat16], "S_out", units=(0,))
    y_g, S_g = strd.ssd_prefill_gather(dev(x), dev(dt), dev(A), dev(B), dev(C), dev(idx), N, M, D=dev(D), S_in=dev(S_in))
    assert torch.equal(y_g, y) and torch.equal(S_g, S), "the gathering scan must give the bits of compact + scan"


@pytest.mark.parametrize("a_scale", [1.0, 1e-3, 0.0])
@pytest.mark.parametrize("T,H,P,G,n", [(1600, 4, 64, 2, 128), (2085, 4, 64, 1, 128), (1100, 6, 96, 2, 64), (1300, 2, 128, 1, 64),
                                       (1500, 4, 64, 2, 64), (1990, 8, 64, 4, 64), (1290, 6, 64, 2, 128)])
def test_ssd_prefill_segments_of_the_sequence(T, H, P, G, n, a_scale):
    """Few heads and a long sequence: the kernel cuts the sequence into segments that run side by
    side and repairs the seams afterwards.  With the workload's A the state at a seam dies within a
    few tokens; with A scaled down, or A = 0 (no decay at all), it reaches across whole segments and
    through several seams.  Dense with D and a carried-in state, and through an index list.  Head sizes of
    64 with an even number of heads per group run two heads per workgroup (both state sizes), the others
    (96, 128 channels; three heads per group) one."""
    _say("ssd_prefill segments T=%d H=%d P=%d G=%d n=%d A x %g" % (T, H, P, G, n, a_scale))
    g = torch.Generator().manual_seed(T + H)
    M = 19
    K = T - M
    N = K + K // 3 + 5
    rows = N + M
    x = torch.randn(rows, H, P, generator=g).to(torch.bfloat16)
    B = (torch.randn(rows, G, n, generator=g) / n ** 0.5).to(torch.bfloat16)
    C = torch.randn(rows, G, n, generator=g).to(torch.bfloat16)
    dt = torch.nn.functional.softplus(torch.randn(rows, H, generator=g))
    A = -torch.exp(2 * torch.rand(H, generator=g)) * a_scale
    D = torch.randn(H, generator=g)
    S_in = torch.randn(H, P, n, generator=g)
    idx = torch.sort(torch.randperm(N, generator=g)[:K]).values.to(torch.int32)
    keep = torch.cat([idx.long(), torch.arange(N, rows)])
    f = synth.np64
    y_ref, S_ref = oracle.ssd_seq(f(x[keep]), f(dt[keep]), f(A), f(B[keep]), f(C[keep]), f(D), f(S_in))
    dev = lambda t: t.to(DEV)
    y, S = strd.ssd_prefill(dev(x[keep].contiguous()), dev(dt[keep].contiguous()), dev(A), dev(B[keep].contiguous()),
                            dev(C[keep].contiguous()), D=dev(D), S_in=dev(S_in))
    assert_close(f(y), y_ref, TOL[torch.bfloat16], "y", units=(1,))
    assert_close(f(S), S_ref, TOL[torch.bfloat16], "S_out", units=(0,))
    y_g, S_g = strd.ssd_prefill_gather(dev(x), dev(dt), dev(A), dev(B), dev(C), dev(idx), N, M, D=dev(D), S_in=dev(S_in))
    assert torch.equal(y_g, y) and torch.equal(S_g, S), "the gathering scan must give the bits of compact + scan"
    # without a state output the seams are repaired all the same
    y2, none = strd.ssd_prefill(dev(x[keep].contiguous()), dev(dt[keep].contiguous()), dev(A), dev(B[keep].contiguous()),
                                dev(C[keep].contiguous()), D=dev(D), S_in=dev(S_in), want_state=False)
    assert none is None and torch.equal(y2, y)


def test_ssd_prefill_split_call_continues_the_scan():
    w = MAMBA_CASES["c2-short"]
    _say("ssd_prefill split call")
    t = _mamba_case(w, seed=11)
    T, cut = 700, 293
    x, dt, B, C = (t[k][:T].contiguous() for k in ("x", "dt", "B", "C"))
    y, S = strd.ssd_prefill(x, dt, t["A"], B, C, chunk=256)
    ya, Sa = strd.ssd_prefill(x[:cut].contiguous(), dt[:cut].contiguous(), t["A"], B[:cut].contiguous(),
                              C[:cut].contiguous(), chunk=256)
    yb, Sb = strd.ssd_prefill(x[cut:].contiguous(), dt[cut:].contiguous(), t["A"], B[cut:].contiguous(),
                              C[cut:].contiguous(), S_in=Sa, chunk=256)
    tol = TOL[torch.bfloat16]
    assert_close(synth.np64(torch.cat([ya, yb])), synth.np64(y), tol, "split y", units=(1,))
    assert_close(synth.np64(Sb), synth.np64(S), tol, "split S", units=(0,))


@pytest.mark.parametrize("name,K,extras", [("c2-short", 375, True), ("c2-short", 1, False), ("c2-short", 0, True),
                                           ("c2-short", 1500, False), ("c2-short", 283, False), ("n64", 130, True)])
def test_ssd_prefill_gather_equals_compact_then_scan(name, K, extras):
    w = MAMBA_CASES[name]
    s = w.mamba
    N, M = w.N, w.M
    _say("ssd_prefill_gather %s N=%d M=%d K=%d" % (name, N, M, K))
    t = _mamba_case(w, seed=K + 3)
    g = torch.Generator(device=DEV).manual_seed(9)
    idx = torch.randperm(N, generator=g, device=DEV)[:K].sort().values.to(torch.int32)
    D = torch.randn(s.H, generator=g, device=DEV) if extras else None
    S_in = torch.randn(s.H, s.P, s.n, generator=g, device=DEV) if extras else None
    y, S = strd.ssd_prefill_gather(t["x"], t["dt"], t["A"], t["B"], t["C"], idx, N, M, D, S_in, chunk=s.chunk)
    xs, dts, Bs, Cs = (strd.compact(t[k], idx, N, M) for k in ("x", "dt", "B", "C"))
    y2, S2 = strd.ssd_prefill(xs, dts, t["A"], Bs, Cs, D, S_in, chunk=s.chunk)
    assert torch.equal(y, y2) and torch.equal(S, S2)  # same arithmetic on the same rows: bit for bit
    idx_np = idx.cpu().numpy()
    yw, Sw = oracle.ssd_seq(*(oracle.compact(synth.np64(t[k]), idx_np, N, M)[0] for k in ("x", "dt")),
                            synth.np64(t["A"]), *(oracle.compact(synth.np64(t[k]), idx_np, N, M)[0] for k in ("B", "C")),
                            None if D is None else synth.np64(D), None if S_in is None else synth.np64(S_in))
    tol = TOL[torch.bfloat16]
    assert_close(synth.np64(y), yw, tol, "gather y", units=(1,))
    assert_close(synth.np64(S), Sw, tol, "gather S_out", units=(0,))


def test_ssd_prefill_gather_refuses_what_the_matrix_core_kernel_does_not_cover():
    w = synth.WORKLOADS["c1"]  # fp32 I/O
    t = _mamba_case(w)
    idx = torch.arange(10, device=DEV, dtype=torch.int32)
    with pytest.raises(strd.StrdError):
        strd.ssd_prefill_gather(t["x"], t["dt"], t["A"], t["B"], t["C"], idx, w.N, w.M)


@pytest.mark.parametrize("name,T", [("c1", 1056), ("c1", 544), ("c3-short", 333), ("c3-short", 1537), ("odd", 100),
                                    ("c1", 1), ("c1", 0), ("d64", 200), ("d64", 705)])
def test_attn_prefill_parity(name, T):
    w = ATTN_CASES[name]
    _say("attn_prefill %s T=%d %s" % (name, T, w.dtype))
    t = _attn_case(w, seed=T)
    q, k, v = (t[n][:T].contiguous() for n in ("q", "k", "v"))
    o = strd.attn_prefill(q, k, v)
    want = oracle.attn(synth.np64(q), synth.np64(k), synth.np64(v))
    assert_close(synth.np64(o), want, TOL[synth.torch_dtype(w.dtype)], "attn o", units=(0, 1))


# Many heads on a short sequence: enough 256-query blocks for the form with 8 computing and 4 copy
# waves, at sizes the oracle still finishes in seconds; 188, 1 and 255 queries in the last block.
WIDE_ATTN = {
    "wide128": synth.shrink(synth.WORKLOADS["c3"], N=800, M=0, d_model=256, attn=synth.AttnShape(Hq=128, Hkv=32, d=128)),
    "wide64": synth.shrink(synth.WORKLOADS["c3"], N=1100, M=0, d_model=256, attn=synth.AttnShape(Hq=192, Hkv=48, d=64)),
}


@pytest.mark.parametrize("name,T", [("wide128", 700), ("wide128", 513), ("wide64", 767), ("wide64", 640), ("wide64", 1025)])
def test_attn_prefill_parity_many_heads(name, T):
    w = WIDE_ATTN[name]
    _say("attn_prefill %s T=%d Hq=%d" % (name, T, w.attn.Hq))
    t = _attn_case(w, seed=T)
    q, k, v = (t[n][:T].contiguous() for n in ("q", "k", "v"))
    o = strd.attn_prefill(q, k, v)
    want = oracle.attn(synth.np64(q), synth.np64(k), synth.np64(v))
    assert_close(synth.np64(o), want, TOL[torch.bfloat16], "attn o", units=(0, 1))


@pytest.mark.parametrize("pattern", ["rising", "falling", "spiky", "flat"])
def test_attn_prefill_lazy_reference_adversarial(pattern):
    """Score patterns that stress the lazily-following softmax reference: a running max that grows at
    every tile (rescale each time), one that never moves after the first key, isolated keys far
    above the rest (jumps of hundreds of log2 units), and all scores equal."""
    _say("attn_prefill adversarial scores: " + pattern)
    T, Hq, Hkv, d = 700, 4, 2, 128
    g = torch.Generator().manual_seed(5)
    u = torch.nn.functional.normalize(torch.randn(d, generator=g), dim=0)
    t = torch.arange(T, dtype=torch.float32)
    if pattern == "rising":
        kmag = 0.05 * t                      # score against q = 30 u grows by 1.5 per key
    elif pattern == "falling":
        kmag = -0.05 * t
    elif pattern == "spiky":
        kmag = torch.zeros(T)
        kmag[37::97] = 12.0                  # 360 above the rest
    else:
        kmag = torch.zeros(T)
    k = (kmag[:, None, None] * u + 0.01 * torch.randn(T, Hkv, d, generator=g)).to(torch.bfloat16)
    q = (30.0 * u + 0.01 * torch.randn(T, Hq, d, generator=g)).to(torch.bfloat16)
    v = torch.randn(T, Hkv, d, generator=g).to(torch.bfloat16)
    o = strd.attn_prefill(q.to(DEV), k.to(DEV), v.to(DEV), scale=1.0)
    want = oracle.attn(synth.np64(q), synth.np64(k), synth.np64(v), scale=1.0)
    assert_close(synth.np64(o), want, TOL[torch.bfloat16], "attn o (%s)" % pattern, units=(0, 1))


# ------------------------------------------------------------------ block glue -------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,d", [(1, 64), (37, 4096), (300, 1000), (0, 128)])
def test_rmsnorm_parity(T, d, dtype):
    _say("rmsnorm T=%d d=%d %s" % (T, d, dtype))
    g = torch.Generator(device=DEV).manual_seed(T + d)
    x = (3 * torch.randn(T, d, generator=g, device=DEV)).to(dtype)
    w = torch.randn(d, generator=g, device=DEV).to(dtype)
    got = strd.rmsnorm(x, w, 1e-5)
    if T:
        assert_close(synth.np64(got), oracle.rmsnorm(synth.np64(x), synth.np64(w), 1e-5), TOL[dtype], "rmsnorm")
        # rows whose mean square is at or below eps: eps decides the result, so its place in the formula shows
        small = (x.float() * 1e-3).to(dtype)
        assert_close(synth.np64(strd.rmsnorm(small, w, 1e-5)), oracle.rmsnorm(synth.np64(small), synth.np64(w), 1e-5),
                     TOL[dtype], "rmsnorm, small rows")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,D,groups", [(5, 64, 1), (33, 8192, 8), (130, 768, 3)])
def test_gated_rmsnorm_parity(T, D, groups, dtype):
    _say("gated_rmsnorm T=%d D=%d groups=%d %s" % (T, D, groups, dtype))
    g = torch.Generator(device=DEV).manual_seed(T + D)
    y = torch.randn(T, D, generator=g, device=DEV).to(dtype)
    wide = (2 * torch.randn(T, D + 40, generator=g, device=DEV)).to(dtype)
    z = wide[:, 24:24 + D]                                  # a column slice: rows of pitch D + 40
    w = torch.randn(D, generator=g, device=DEV).to(dtype)
    got = strd.gated_rmsnorm(y, z, w, groups, 1e-5)
    want = oracle.gated_rmsnorm(synth.np64(y), synth.np64(z.contiguous()), synth.np64(w), groups, 1e-5)
    assert_close(synth.np64(got), want, TOL[dtype], "gated_rmsnorm")
    y_small = (y.float() * 2e-3).to(dtype)                  # groups whose mean square is near eps
    got = strd.gated_rmsnorm(y_small, z, w, groups, 1e-5)
    want = oracle.gated_rmsnorm(synth.np64(y_small), synth.np64(z.contiguous()), synth.np64(w), groups, 1e-5)
    assert_close(synth.np64(got), want, TOL[dtype], "gated_rmsnorm, small rows")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,Cx,Cb,W,extra", [(1, 8, 8, 4, 0), (50, 64, 16, 4, 8), (300, 256, 128, 4, 24), (17, 32, 8, 2, 0),
                                             (9, 16, 8, 1, 0)])
def test_conv1d_silu_parity(T, Cx, Cb, W, extra, dtype):
    _say("conv1d_silu T=%d Cx=%d Cb=%d W=%d %s" % (T, Cx, Cb, W, dtype))
    g = torch.Generator(device=DEV).manual_seed(T + Cx)
    Ct = Cx + 2 * Cb
    wide = torch.randn(T, Ct + extra, generator=g, device=DEV).to(dtype)   # trailing columns (dt) are not touched
    w = (0.5 * torch.randn(Ct, W, generator=g, device=DEV)).to(dtype)
    b = torch.randn(Ct, generator=g, device=DEV).to(dtype)
    x, B, C = strd.conv1d_silu(wide, w, b, Cx, Cb)
    want = oracle.conv1d_silu(synth.np64(wide[:, :Ct].contiguous()), synth.np64(w), synth.np64(b))
    tol = TOL[dtype]
    assert_close(synth.np64(x), want[:, :Cx], tol, "conv x")
    assert_close(synth.np64(B), want[:, Cx:Cx + Cb], tol, "conv B")
    assert_close(synth.np64(C), want[:, Cx + Cb:], tol, "conv C")
    x2, _, _ = strd.conv1d_silu(wide, w, None, Cx, Cb)
    assert_close(synth.np64(x2), oracle.conv1d_silu(synth.np64(wide[:, :Ct].contiguous()), synth.np64(w))[:, :Cx], tol,
                 "conv without bias")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_softplus_dt_parity(dtype):
    _say("softplus_dt %s" % dtype)
    g = torch.Generator(device=DEV).manual_seed(3)
    wide = (6 * torch.randn(77, 200, generator=g, device=DEV)).to(dtype)
    raw = wide[:, 72:200]
    bias = torch.randn(128, generator=g, device=DEV)
    got = strd.softplus_dt(raw, bias)
    want = oracle.softplus_dt(synth.np64(raw.contiguous()), synth.np64(bias))
    assert_close(got.cpu().numpy().astype(np.float64), want, 1e-5, "softplus_dt")
    assert (got > 0).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,Kd,Nd", [(1, 64, 8), (37, 300, 129), (256, 1024, 2048)])
def test_linear_parity(T, Kd, Nd, dtype):
    _say("linear T=%d Kd=%d Nd=%d %s" % (T, Kd, Nd, dtype))
    g = torch.Generator(device=DEV).manual_seed(T + Kd)
    x = torch.randn(T, Kd, generator=g, device=DEV).to(dtype)
    w = (torch.randn(Kd, Nd, generator=g, device=DEV) / Kd ** 0.5).to(dtype)
    r = torch.randn(T, Nd, generator=g, device=DEV).to(dtype)
    tol = TOL[dtype]
    assert_close(synth.np64(strd.linear(x, w)), synth.np64(x) @ synth.np64(w), tol, "linear")
    assert_close(synth.np64(strd.linear(x, w, r)), synth.np64(x) @ synth.np64(w) + synth.np64(r), tol, "linear + residual")
    acc = r.clone()
    strd.linear(x, w, acc, out=acc)                       # residual stream updated in place
    assert_close(synth.np64(acc), synth.np64(x) @ synth.np64(w) + synth.np64(r), tol, "linear in place")


@pytest.mark.parametrize("T,Kd,Nd", [(1, 64, 8), (37, 320, 136), (300, 64, 264), (257, 128, 24), (40, 192, 512), (513, 1024, 2056),
                                     (2049, 512, 520)])
def test_linear_mfma_parity(T, Kd, Nd):
    """The library's own projection kernel against the dense product in fp64: one tile and several, ragged
    last token and column tiles, every length of the copy ring's start-up and tail (2, 4, 6 stages of 32 and
    more), the residual separately and in place."""
    _say("linear_mfma T=%d Kd=%d Nd=%d" % (T, Kd, Nd))
    g = torch.Generator(device=DEV).manual_seed(3 * T + Kd)
    dtype = torch.bfloat16
    x = torch.randn(T, Kd, generator=g, device=DEV).to(dtype)
    w = (torch.randn(Kd, Nd, generator=g, device=DEV) / Kd ** 0.5).to(dtype)
    r = torch.randn(T, Nd, generator=g, device=DEV).to(dtype)
    want = synth.np64(x) @ synth.np64(w)
    tol = TOL[dtype]
    out = torch.full((T + 1, Nd), 7.0, dtype=dtype, device=DEV)       # one guard row after the output
    strd.linear_mfma(x, w, out=out[:T])
    assert_close(synth.np64(out[:T]), want, tol, "linear_mfma")
    assert (out[T] == 7.0).all(), "wrote past the last token"
    assert_close(synth.np64(strd.linear_mfma(x, w, r)), want + synth.np64(r), tol, "linear_mfma + residual")
    acc = r.clone()
    strd.linear_mfma(x, w, acc, out=acc)                               # residual stream updated in place
    assert_close(synth.np64(acc), want + synth.np64(r), tol, "linear_mfma in place")
    # one rounding after fp32 accumulation: within one bf16 step of the exact value, element by element
    got = synth.np64(strd.linear_mfma(x, w))
    assert (np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-3).all()


def test_linear_picks_its_kernel_by_size_and_both_agree():
    """strd_linear runs the library's own kernel from one 256 x 256 output tile per CU up and rocBLAS below;
    both paths against the dense product in fp64 on a shape of 17 x 16 tiles, with the residual in place."""
    T, Kd, Nd = 4352, 256, 4096
    _say("linear dispatch T=%d Kd=%d Nd=%d" % (T, Kd, Nd))
    g = torch.Generator(device=DEV).manual_seed(11)
    x = torch.randn(T, Kd, generator=g, device=DEV).to(torch.bfloat16)
    w = (torch.randn(Kd, Nd, generator=g, device=DEV) / Kd ** 0.5).to(torch.bfloat16)
    r = torch.randn(T, Nd, generator=g, device=DEV).to(torch.bfloat16)
    want = synth.np64(x) @ synth.np64(w) + synth.np64(r)
    tol = TOL[torch.bfloat16]
    for name, fn in (("linear", strd.linear), ("linear_mfma", strd.linear_mfma), ("linear_library", strd.linear_library)):
        acc = r.clone()
        fn(x, w, acc, out=acc)
        assert_close(synth.np64(acc), want, tol, name)
    # the dispatching call and the own kernel are the same launch: identical bits
    assert torch.equal(strd.linear(x, w, r), strd.linear_mfma(x, w, r))


def test_glue_refuses_misaligned_or_inconsistent_arguments():
    x = torch.randn(8, 30, device=DEV, dtype=torch.bfloat16)
    with pytest.raises(strd.StrdError):
        strd.conv1d_silu(x, torch.randn(20, 4, device=DEV, dtype=torch.bfloat16), None, 12, 4)   # not multiples of 8
    with pytest.raises(strd.StrdError):
        strd.gated_rmsnorm(x, x, torch.randn(30, device=DEV, dtype=torch.bfloat16), groups=4)     # 30 % 4 != 0


# ------------------------------------------------------------------ whole reduced layer ----
def _reduced_mamba_layer_dev(t, N, M, K, chunk):
    s = strd.score_mamba(t["B"][:N].contiguous(), t["C"][N:].contiguous(), t["dt"][:N].contiguous())
    idx = strd.select_topk(s, K)
    xs = strd.compact(t["x"], idx, N, M)
    Bs = strd.compact(t["B"], idx, N, M)
    Cs = strd.compact(t["C"], idx, N, M)
    dts, pos = strd.compact(t["dt"], idx, N, M, want_pos=True)
    y, S = strd.ssd_prefill(xs, dts, t["A"], Bs, Cs, chunk=chunk)
    return s, idx, pos, y, S


def test_reduced_mamba_layer_tiny_pair_matches_oracle_chain():
    w = synth.WORKLOADS["c1"]
    _say("reduced mamba layer c1")
    t = _mamba_case(w)
    N, M, K = w.N, w.M, w.K
    s, idx, pos, y, S = _reduced_mamba_layer_dev(t, N, M, K, w.mamba.chunk)
    s_ref = oracle.score_mamba(synth.np64(t["B"][:N]), synth.np64(t["C"][N:]), synth.np64(t["dt"][:N]))
    assert_close(s.cpu().numpy(), s_ref, 1e-4, "score", units=(0,))
    swaps = assert_topk_equivalent(idx.cpu().numpy(), s_ref, K, 1e-4)
    # the mixer is checked on the device's own selection (identical to the oracle's unless a near-tie swapped)
    idx_np = idx.cpu().numpy()
    xs, pos_ref = oracle.compact(synth.np64(t["x"]), idx_np, N, M)
    np.testing.assert_array_equal(pos.cpu().numpy(), pos_ref)
    yw, Sw = oracle.ssd_seq(xs, oracle.compact(synth.np64(t["dt"]), idx_np, N, M)[0], synth.np64(t["A"]),
                            oracle.compact(synth.np64(t["B"]), idx_np, N, M)[0],
                            oracle.compact(synth.np64(t["C"]), idx_np, N, M)[0])
    assert_close(synth.np64(y), yw, 1e-4, "reduced y", units=(1,))
    assert_close(synth.np64(S), Sw, 1e-4, "reduced S", units=(0,))
    _say("near-tie swaps vs oracle: %d" % swaps)


def test_reduced_attention_layer_tiny_pair_matches_oracle_chain():
    w = synth.WORKLOADS["c1"]
    _say("reduced attention layer c1")
    t = _attn_case(w)
    N, M, K = w.N, w.M, w.K
    s = strd.score_attn(t["q"][N:].contiguous(), t["k"][:N].contiguous())
    idx = strd.select_topk(s, K)
    qs, ks, vs = (strd.compact(t[n], idx, N, M) for n in ("q", "k", "v"))
    o = strd.attn_prefill(qs, ks, vs)
    s_ref = oracle.score_attn(synth.np64(t["q"][N:]), synth.np64(t["k"][:N]))
    assert_close(s.cpu().numpy(), s_ref, 1e-4, "score", units=(0,))
    assert_topk_equivalent(idx.cpu().numpy(), s_ref, K, 1e-4)
    idx_np = idx.cpu().numpy()
    want = oracle.attn(*(oracle.compact(synth.np64(t[n]), idx_np, N, M)[0] for n in ("q", "k", "v")))
    assert_close(synth.np64(o), want, 1e-4, "reduced o", units=(0, 1))


def test_full_budget_reproduces_the_unreduced_layer_on_device():
    w = synth.WORKLOADS["c1"]
    _say("100% budget identity c1")
    t = _mamba_case(w)
    N, M = w.N, w.M
    s, idx, pos, y, S = _reduced_mamba_layer_dev(t, N, M, N, w.mamba.chunk)
    assert torch.equal(idx.cpu(), torch.arange(N, dtype=torch.int32))
    assert torch.equal(pos.cpu(), torch.arange(N + M, dtype=torch.int32))
    y_full, S_full = strd.ssd_prefill(t["x"], t["dt"], t["A"], t["B"], t["C"], chunk=w.mamba.chunk)
    assert torch.equal(y, y_full) and torch.equal(S, S_full)


# ------------------------------------------------------------------ error behaviour --------
def test_invalid_arguments_are_refused_without_launching():
    _say("error paths")
    s = torch.rand(100, device=DEV)
    with pytest.raises(strd.StrdError):
        strd.select_topk(s, 0)
    with pytest.raises(strd.StrdError):
        strd.select_topk(s, 101)
    q = torch.randn(4, 3, 8, device=DEV)
    k = torch.randn(9, 2, 8, device=DEV)
    with pytest.raises(strd.StrdError):
        strd.score_attn(q, k)          # 3 query heads over 2 kv heads
    torch.cuda.synchronize()
