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
    assert_close(f(y), y_ref, TOL[torch.bfloat16], "y")
    assert_close(f(S), S_ref, TOL[torch.bfloat16], "S")
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
    assert_close(f(o[rows]), oracle.attn(f(q), f(k), f(v), rows=rows), TOL[torch.bfloat16], "o")


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
    assert_close(s.cpu().numpy(), oracle.score_mamba(f(Bv), f(Ct), f(dtv)), TOL[torch.bfloat16], "score_mamba")
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
    assert_close(sa.cpu().numpy(), oracle.score_attn(f(qt), f(kv)), TOL[torch.bfloat16], "score_attn")
