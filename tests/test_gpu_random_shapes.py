"""Parity of the HIP library with the CPU fp64 oracle on seeded random shapes: head counts, head
sizes, state sizes, group counts and ragged token counts drawn together, so that combinations the
hand-picked cases of the other parity tests do not list are exercised too.  Needs a GPU."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_00198_amd as strd
from paper_2603_00198_amd import synth
from util import TOL, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda"
f = synth.np64
SEEDS = list(range(12))


def _say(msg):
    print("[case] " + msg, flush=True)


def _dev(t):
    return t.to(DEV)


@pytest.mark.parametrize("seed", SEEDS)
def test_ssd_prefill_random_shape(seed):
    """Dense scan against the sequential recurrence (Eq. 1 with the discretisation of Sec. 3.1), and
    the gather form against the dense one bit for bit."""
    rng = np.random.default_rng(1000 + seed)
    g = torch.Generator().manual_seed(1000 + seed)
    H = int(rng.choice([1, 2, 3, 8]))
    G = int(rng.choice([d for d in (1, 2, 3, 8) if H % d == 0]))
    P = int(rng.choice([32, 64, 96]))
    n = int(rng.choice([64, 128]))
    T = int(rng.integers(1, 700))
    M = int(rng.integers(1, min(T, 40) + 1))
    K = T - M
    N = K + int(rng.integers(0, 300))
    rows = N + M
    _say("ssd_prefill random H=%d G=%d P=%d n=%d T=%d K=%d N=%d" % (H, G, P, n, T, K, N))
    x = torch.randn(rows, H, P, generator=g).to(torch.bfloat16)
    B = (torch.randn(rows, G, n, generator=g) / n ** 0.5).to(torch.bfloat16)
    C = torch.randn(rows, G, n, generator=g).to(torch.bfloat16)
    dt = torch.nn.functional.softplus(torch.randn(rows, H, generator=g))
    A = -torch.exp(2 * torch.rand(H, generator=g))
    S_in = torch.randn(H, P, n, generator=g)
    idx = torch.sort(torch.randperm(N, generator=g)[:K]).values.to(torch.int32)
    keep = torch.cat([idx.long(), torch.arange(N, rows)])
    y_ref, S_ref = oracle.ssd_seq(f(x[keep]), f(dt[keep]), f(A), f(B[keep]), f(C[keep]), None, f(S_in))
    y, S = strd.ssd_prefill(_dev(x[keep].contiguous()), _dev(dt[keep].contiguous()), _dev(A),
                            _dev(B[keep].contiguous()), _dev(C[keep].contiguous()), S_in=_dev(S_in))
    assert_close(f(y), y_ref, TOL[torch.bfloat16], "y", units=(1,))
    assert_close(f(S), S_ref, TOL[torch.bfloat16], "S", units=(0,))
    yg, Sg = strd.ssd_prefill_gather(_dev(x), _dev(dt), _dev(A), _dev(B), _dev(C), _dev(idx), N, M, S_in=_dev(S_in))
    assert torch.equal(yg, y) and torch.equal(Sg, S)


@pytest.mark.parametrize("seed", SEEDS)
def test_attn_prefill_random_shape(seed):
    """Causal grouped-query attention (Sec. 3.1), sampled rows against the oracle; the head and
    token counts land on either side of the switch between the two kernel forms."""
    rng = np.random.default_rng(2000 + seed)
    g = torch.Generator().manual_seed(2000 + seed)
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 8, 24]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 8]))
    T = int(rng.integers(1, 900 if Hq <= 16 else 600))
    _say("attn_prefill random T=%d Hq=%d Hkv=%d d=%d" % (T, Hq, Hkv, d))
    q = torch.randn(T, Hq, d, generator=g).to(torch.bfloat16)
    k = torch.randn(T, Hkv, d, generator=g).to(torch.bfloat16)
    v = torch.randn(T, Hkv, d, generator=g).to(torch.bfloat16)
    o = strd.attn_prefill(_dev(q), _dev(k), _dev(v))
    rows = sorted(set(int(r) for r in rng.integers(0, T, 24)) | {0, T - 1})
    assert_close(f(o[rows]), oracle.attn(f(q), f(k), f(v), rows=rows), TOL[torch.bfloat16], "o", units=(0, 1))


# N, M, G, H, n: sequences long enough for the kernel that keeps a group's text rows in LDS -- one
# and two token blocks per wave, ragged token and text counts, more text rows than fit LDS at once
# (two passes), head counts per group other than 16, a single group
LONG_SCORE_CASES = [
    (16411, 37, 8, 128, 128),
    (40000, 200, 8, 128, 128),
    (17000, 600, 8, 128, 128),
    (16500, 1300, 8, 128, 128),   # three passes over the text rows
    (33001, 1150, 8, 24, 64),
    (66000, 129, 2, 32, 128),
    (131075, 64, 1, 4, 64),
    (140000, 96, 8, 64, 64),
]


@pytest.mark.parametrize("N,M,G,H,n", LONG_SCORE_CASES)
def test_score_mamba_long_sequences(N, M, G, H, n):
    """Eq. 4 (Decoupled Content Alignment) on long sequences, every token against the oracle."""
    g = torch.Generator().manual_seed(N + M)
    _say("score_mamba long N=%d M=%d G=%d H=%d n=%d" % (N, M, G, H, n))
    Bv = (torch.randn(N, G, n, generator=g) / n ** 0.5).to(torch.bfloat16)
    Ct = torch.randn(M, G, n, generator=g).to(torch.bfloat16)
    dtv = torch.nn.functional.softplus(torch.randn(N, H, generator=g))
    s = strd.score_mamba(_dev(Bv), _dev(Ct), _dev(dtv))
    assert_close(s.cpu().numpy(), oracle.score_mamba(f(Bv), f(Ct), f(dtv)), TOL[torch.bfloat16], "score_mamba", units=(0,))


@pytest.mark.parametrize("seed", SEEDS)
def test_scores_and_selection_random_shape(seed):
    """Both scores (Eq. 3 and Eq. 4) against the oracle, and the selection on the device's own
    scores against the oracle's selection on the same numbers, index for index."""
    rng = np.random.default_rng(3000 + seed)
    g = torch.Generator().manual_seed(3000 + seed)
    N = int(rng.integers(1, 5000))
    M = int(rng.integers(1, 200))
    G = int(rng.choice([1, 2, 8]))
    H = G * int(rng.choice([1, 4, 16]))
    n = int(rng.choice([64, 128]))
    _say("score_mamba random N=%d M=%d G=%d H=%d n=%d" % (N, M, G, H, n))
    Bv = (torch.randn(N, G, n, generator=g) / n ** 0.5).to(torch.bfloat16)
    Ct = torch.randn(M, G, n, generator=g).to(torch.bfloat16)
    dtv = torch.nn.functional.softplus(torch.randn(N, H, generator=g))
    s = strd.score_mamba(_dev(Bv), _dev(Ct), _dev(dtv))
    assert_close(s.cpu().numpy(), oracle.score_mamba(f(Bv), f(Ct), f(dtv)), TOL[torch.bfloat16], "score_mamba", units=(0,))
    K = int(rng.integers(1, N + 1))
    got = strd.select_topk(s, K).cpu().numpy()
    np.testing.assert_array_equal(got, oracle.select_topk(s.cpu().numpy().astype(np.float64), K))

    Hkv = int(rng.choice([1, 2, 4]))
    Hq = Hkv * int(rng.choice([1, 2, 4]))
    d = int(rng.choice([64, 128]))
    _say("score_attn random N=%d M=%d Hq=%d Hkv=%d d=%d" % (N, M, Hq, Hkv, d))
    qt = torch.randn(M, Hq, d, generator=g).to(torch.bfloat16)
    kv = torch.randn(N, Hkv, d, generator=g).to(torch.bfloat16)
    sa = strd.score_attn(_dev(qt), _dev(kv))
    assert_close(sa.cpu().numpy(), oracle.score_attn(f(qt), f(kv)), TOL[torch.bfloat16], "score_attn", units=(0,))


def _bits(t):
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


@pytest.mark.parametrize("seed", SEEDS)
def test_compact_random_shape(seed):
    """Compaction (Sec. 3.1: the retained tokens keep their order and positions), bit for bit, for
    row sizes that are and are not multiples of 16 bytes, one tensor and several in one launch."""
    rng = np.random.default_rng(4000 + seed)
    g = torch.Generator().manual_seed(4000 + seed)
    N = int(rng.integers(1, 4000))
    M = int(rng.integers(0, 100))
    K = int(rng.integers(0, N + 1))
    count = int(rng.integers(1, 6))
    shapes = []
    for _ in range(count):        # rows are whole 4-byte words: an even element count for bf16
        dtype = torch.bfloat16 if rng.integers(2) else torch.float32
        elems = [2, 6, 8, 24, 130, 256, 1000, 4096] if dtype == torch.bfloat16 else [1, 2, 7, 8, 24, 65, 256, 1000, 4096]
        shapes.append((int(rng.choice(elems)), dtype))
    _say("compact random N=%d M=%d K=%d rows=%s" % (N, M, K, [(e, str(d)) for e, d in shapes]))
    srcs = [torch.randn(N + M, e, generator=g).to(d) for e, d in shapes]
    idx = torch.sort(torch.randperm(N, generator=g)[:K]).values.to(torch.int32)
    pos_in = torch.randperm(3 * (N + M), generator=g)[: N + M].to(torch.int32)
    outs, pos = strd.compact_batch([_dev(t) for t in srcs], _dev(idx), N, M, pos_in=_dev(pos_in))
    for t, o in zip(srcs, outs):
        want, want_pos = oracle.compact(_bits(t).numpy(), idx.numpy(), N, M, pos_in=pos_in.numpy())
        np.testing.assert_array_equal(_bits(o.cpu()).numpy(), want)
        np.testing.assert_array_equal(pos.cpu().numpy(), want_pos)
    one, pos1 = strd.compact(_dev(srcs[0]), _dev(idx), N, M, pos_in=_dev(pos_in))
    assert torch.equal(one, outs[0]) and torch.equal(pos1, pos)


@pytest.mark.parametrize("seed", SEEDS)
def test_avgpool_random_shape(seed):
    """The average-pool baseline (Sec. 4.1) for window sizes from 1 row to the whole sequence."""
    rng = np.random.default_rng(5000 + seed)
    g = torch.Generator().manual_seed(5000 + seed)
    N = int(rng.integers(1, 3000))
    M = int(rng.integers(0, 60))
    K = int(rng.integers(1, N + 1)) if rng.integers(3) else int(rng.integers(1, min(N, 8) + 1))
    D = int(rng.choice([7, 8, 24, 136, 256, 1024]))
    dtype = torch.bfloat16 if rng.integers(2) else torch.float32
    _say("avgpool random N=%d M=%d K=%d D=%d %s" % (N, M, K, D, dtype))
    src = torch.randn(N + M, D, generator=g).to(dtype)
    pos_in = torch.randperm(3 * (N + M), generator=g)[: N + M].to(torch.int32)
    dst, pos = strd.avgpool(_dev(src), N, M, K, pos_in=_dev(pos_in))
    want, want_pos = oracle.avgpool(f(src), N, M, K, pos_in.numpy())
    np.testing.assert_array_equal(pos.cpu().numpy(), want_pos)
    assert_close(f(dst), want, TOL[dtype], "avgpool")
    assert torch.equal(dst[K:].cpu(), src[N:])


@pytest.mark.parametrize("seed", SEEDS)
def test_decode_steps_random_shape(seed):
    """One token of the recurrence (Eq. 1) and of causal attention over a cache (Sec. 3.1)."""
    rng = np.random.default_rng(6000 + seed)
    g = torch.Generator().manual_seed(6000 + seed)
    dtype = torch.bfloat16 if rng.integers(2) else torch.float32
    G = int(rng.choice([1, 2, 3]))
    H = G * int(rng.choice([1, 2, 4]))
    P = int(rng.choice([3, 5, 32, 64]))
    n = int(rng.choice([10, 16, 64, 128, 200]))
    _say("ssd_decode_step random H=%d P=%d G=%d n=%d %s" % (H, P, G, n, dtype))
    x = torch.randn(H, P, generator=g).to(dtype)
    dt = torch.nn.functional.softplus(torch.randn(H, generator=g))
    A = -torch.exp(2 * torch.rand(H, generator=g))
    B = torch.randn(G, n, generator=g).to(dtype)
    C = torch.randn(G, n, generator=g).to(dtype)
    D = torch.randn(H, generator=g) if rng.integers(2) else None
    S = torch.randn(H, P, n, generator=g)
    S_dev = _dev(S)
    y = strd.ssd_decode_step(_dev(x), _dev(dt), _dev(A), _dev(B), _dev(C), None if D is None else _dev(D), S_dev)
    y_ref, S_ref = oracle.ssd_decode_step(f(x), f(dt), f(A), f(B), f(C), None if D is None else f(D), f(S))
    assert_close(f(S_dev), S_ref, 1e-5, "state")
    assert_close(f(y), y_ref, TOL[dtype], "y", units=(0,))

    T = int(rng.integers(1, 20000))
    Hkv = int(rng.choice([1, 2, 8]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 8]))
    d = int(rng.choice([64, 128]))
    _say("attn_decode_step random T=%d Hq=%d Hkv=%d d=%d %s" % (T, Hq, Hkv, d, dtype))
    q = torch.randn(Hq, d, generator=g).to(dtype)
    k = torch.randn(T, Hkv, d, generator=g).to(dtype)
    v = torch.randn(T, Hkv, d, generator=g).to(dtype)
    o = strd.attn_decode_step(_dev(q), _dev(k), _dev(v))
    assert_close(f(o), oracle.attn_decode_step(f(q), f(k), f(v)), TOL[dtype], "attn_decode_step", units=(0,))


@pytest.mark.parametrize("seed", SEEDS)
def test_score_mamba_full_random_shape(seed):
    """The decayed Mamba score (Eq. 3 with the decay of Eq. 2 kept) for mild and strong decay."""
    rng = np.random.default_rng(7000 + seed)
    g = torch.Generator().manual_seed(7000 + seed)
    N = int(rng.integers(1, 3000))
    M = int(rng.integers(1, 100))
    G = int(rng.choice([1, 2, 8]))
    H = G * int(rng.choice([1, 4, 16]))
    n = int(rng.choice([64, 128]))
    a_scale = float(rng.choice([1.0, 0.05, 0.003]))
    _say("score_mamba_full random N=%d M=%d G=%d H=%d n=%d A x %g" % (N, M, G, H, n, a_scale))
    Ball = (torch.randn(N + M, G, n, generator=g) / n ** 0.5).to(torch.bfloat16)
    Call = torch.randn(N + M, G, n, generator=g).to(torch.bfloat16)
    dt = torch.nn.functional.softplus(torch.randn(N + M, H, generator=g) - 2)
    A = -torch.exp(2 * torch.rand(H, generator=g)) * a_scale
    got = strd.score_mamba_full(_dev(Ball[:N].contiguous()), _dev(Call[N:].contiguous()), _dev(dt), _dev(A))
    want = oracle.score_mamba_full(f(Ball), f(Call), f(dt), f(A), N)
    assert_close(got.cpu().numpy(), want, TOL[torch.bfloat16], "score_mamba_full", units=(0,))


@pytest.mark.parametrize("seed", SEEDS)
def test_linear_mfma_random_shape(seed):
    """The library's own projection kernel on token counts, input widths (multiples of 64) and output
    widths (multiples of 8) drawn together: ragged last tiles in both directions, any number of
    k stages, with and without the residual.  Checked against the dense product in fp64."""
    rng = np.random.default_rng(8000 + seed)
    g = torch.Generator().manual_seed(8000 + seed)
    T = int(rng.integers(1, 1400))
    Kd = 64 * int(rng.integers(1, 20))
    Nd = 8 * int(rng.integers(1, 130))
    with_res = bool(rng.integers(2))
    _say("linear_mfma random T=%d Kd=%d Nd=%d residual=%s" % (T, Kd, Nd, with_res))
    assert strd.linear_mfma_supported(T, Kd, Nd, torch.bfloat16)
    x = torch.randn(T, Kd, generator=g).to(torch.bfloat16)
    w = (torch.randn(Kd, Nd, generator=g) / Kd ** 0.5).to(torch.bfloat16)
    r = torch.randn(T, Nd, generator=g).to(torch.bfloat16) if with_res else None
    want = f(x) @ f(w) + (f(r) if with_res else 0.0)
    out = torch.full((T + 1, Nd), 7.0, dtype=torch.bfloat16, device=DEV)      # one guard row after the output
    strd.linear_mfma(_dev(x), _dev(w), _dev(r) if with_res else None, out=out[:T])
    assert_close(f(out[:T]), want, TOL[torch.bfloat16], "linear_mfma")
    assert (out[T] == 7.0).all(), "wrote past the last token"
    # the dispatching call gives the same values whichever kernel it picks (rocBLAS at these sizes)
    assert_close(f(strd.linear(_dev(x), _dev(w), _dev(r) if with_res else None)), want, TOL[torch.bfloat16], "linear")
