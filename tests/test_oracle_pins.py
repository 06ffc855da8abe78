"""Pins for the CPU fp64 oracle: closed forms, independent formulations, library
routines and brute force, chosen so that a dropped term, wrong sign or index, or a
transposed operand in ``oracle/strd_oracle.c`` fails at least one of them.  CPU only."""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle

RNG = np.random.default_rng(1234)


def _ssd_case(T, H, P, G, n, seed=0, with_D=True, with_S=True):
    r = np.random.default_rng(seed)
    x = r.standard_normal((T, H, P))
    dt = np.log1p(np.exp(r.standard_normal((T, H))))
    A = -np.exp(r.uniform(0, 2, H))
    B = r.standard_normal((T, G, n))
    C = r.standard_normal((T, G, n))
    D = r.standard_normal(H) if with_D else None
    S = r.standard_normal((H, P, n)) if with_S else None
    return x, dt, A, B, C, D, S


# ---------------------------------------------------------------- SSD ----

def test_ssd_hand_worked_two_tokens(golden_dir):
    gold = {}
    for line in open(os.path.join(golden_dir, "ssd_two_token.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            gold[k] = float(v)
    x = np.array([3.0, -1.0]).reshape(2, 1, 1)
    dt = np.array([0.5, 2.0]).reshape(2, 1)
    A = np.array([-1.0])
    B = np.array([[1.0, 2.0], [0.5, -1.0]]).reshape(2, 1, 2)
    C = np.array([[1.0, 1.0], [2.0, 0.5]]).reshape(2, 1, 2)
    for fn in (oracle.ssd_seq, lambda *a: oracle.ssd_chunked(*a, chunk=1),
               lambda *a: oracle.ssd_chunked(*a, chunk=2)):
        y, S = fn(x, dt, A, B, C)
        assert y[0, 0, 0] == pytest.approx(gold["y0"], rel=1e-14)
        assert y[1, 0, 0] == pytest.approx(gold["y1"], rel=1e-13)
        assert S[0, 0, 0] == pytest.approx(gold["S1_0"], rel=1e-13)
        assert S[0, 0, 1] == pytest.approx(gold["S1_1"], rel=1e-13)
    y = oracle.ssd_unrolled(x, dt, A, B, C)
    assert y[1, 0, 0] == pytest.approx(gold["y1"], rel=1e-13)


@pytest.mark.parametrize("T,chunk", [(1, 4), (37, 5), (64, 64), (70, 64), (96, 256)])
def test_ssd_three_formulations_agree(T, chunk):
    x, dt, A, B, C, D, S = _ssd_case(T, H=4, P=3, G=2, n=5, seed=T)
    y1, s1 = oracle.ssd_seq(x, dt, A, B, C, D, S)
    y2 = oracle.ssd_unrolled(x, dt, A, B, C, D, S)
    y3, s3 = oracle.ssd_chunked(x, dt, A, B, C, D, S, chunk=chunk)
    np.testing.assert_allclose(y2, y1, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(y3, y1, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(s3, s1, rtol=1e-10, atol=1e-11)


def test_ssd_no_decay_is_prefix_sum():
    T, P = 19, 4
    x = RNG.standard_normal((T, 1, P))
    dt = np.ones((T, 1))
    A = np.zeros(1)
    B = np.zeros((T, 1, 3)); B[:, 0, 0] = 1.0
    C = B.copy()
    for y in (oracle.ssd_seq(x, dt, A, B, C)[0], oracle.ssd_chunked(x, dt, A, B, C, chunk=4)[0],
              oracle.ssd_unrolled(x, dt, A, B, C)):
        np.testing.assert_allclose(y[:, 0, :], np.cumsum(x[:, 0, :], axis=0), rtol=1e-12)


def test_ssd_constant_decay_geometric_series():
    T, a = 25, 0.8
    x = np.ones((T, 1, 1))
    dt = np.ones((T, 1))
    A = np.array([np.log(a)])
    B = np.ones((T, 1, 1)); C = np.ones((T, 1, 1))
    want = (1 - a ** (np.arange(T) + 1)) / (1 - a)
    np.testing.assert_allclose(oracle.ssd_seq(x, dt, A, B, C)[0][:, 0, 0], want, rtol=1e-12)
    np.testing.assert_allclose(oracle.ssd_chunked(x, dt, A, B, C, chunk=7)[0][:, 0, 0], want, rtol=1e-12)


def test_ssd_state_is_outer_product_layout():
    # one token, S_0 = 0: S = x (dt b)^T with shape [P, n] -- catches a transposed state
    x = np.array([2.0, 3.0, 5.0]).reshape(1, 1, 3)
    dt = np.array([[0.5]]); A = np.array([-1.0])
    B = np.array([7.0, 11.0]).reshape(1, 1, 2); C = np.array([1.0, 0.0]).reshape(1, 1, 2)
    y, S = oracle.ssd_seq(x, dt, A, B, C)
    np.testing.assert_allclose(S[0], np.outer([2, 3, 5], [3.5, 5.5]))
    np.testing.assert_allclose(y[0, 0], [7.0, 10.5, 17.5])


def test_ssd_group_mapping_is_block_of_heads():
    # H=4, G=2: heads 0,1 read group 0; heads 2,3 read group 1
    T = 6
    x, dt, A, B, C, _, _ = _ssd_case(T, H=4, P=2, G=2, n=3, seed=5, with_D=False, with_S=False)
    y, _ = oracle.ssd_seq(x, dt, A, B, C)
    for h in range(4):
        g = h // 2
        yh, _ = oracle.ssd_seq(x[:, h:h + 1], dt[:, h:h + 1], A[h:h + 1], B[:, g:g + 1], C[:, g:g + 1])
        np.testing.assert_allclose(y[:, h], yh[:, 0], rtol=1e-13)


def test_ssd_split_call_equals_single_call():
    x, dt, A, B, C, D, S = _ssd_case(50, H=2, P=3, G=1, n=4, seed=9)
    y, s = oracle.ssd_seq(x, dt, A, B, C, D, S)
    ya, sa = oracle.ssd_seq(x[:21], dt[:21], A, B[:21], C[:21], D, S)
    yb, sb = oracle.ssd_seq(x[21:], dt[21:], A, B[21:], C[21:], D, sa)
    np.testing.assert_allclose(np.concatenate([ya, yb]), y, rtol=1e-12)
    np.testing.assert_allclose(sb, s, rtol=1e-12)


def test_ssd_D_is_a_skip_connection():
    x, dt, A, B, C, D, S = _ssd_case(9, H=2, P=3, G=1, n=4, seed=3)
    y0, _ = oracle.ssd_seq(x, dt, A, B, C, None, S)
    y1, _ = oracle.ssd_seq(x, dt, A, B, C, D, S)
    np.testing.assert_allclose(y1 - y0, D[None, :, None] * x, rtol=1e-10, atol=1e-12)


# -------------------------------------------------------- Mamba score ----

def test_score_mamba_scalar_case():
    N, n = 7, 5
    B = RNG.standard_normal((N, 1, n)); C = RNG.standard_normal((1, 1, n))
    dt = RNG.uniform(0.1, 2, (N, 1))
    want = dt[:, 0] * np.abs(B[:, 0] @ C[0, 0])
    np.testing.assert_allclose(oracle.score_mamba(B, C, dt), want, rtol=1e-13)


def test_score_mamba_abs_before_sum_and_head_mean():
    # two text rows with opposite-sign alignments must not cancel
    B = np.array([1.0, 0.0]).reshape(1, 1, 2)
    C = np.array([[2.0, 0.0], [-2.0, 0.0]]).reshape(2, 1, 2)
    dt = np.array([[1.0, 3.0]])           # H=2 heads in one group: mean dt = 2
    assert oracle.score_mamba(B, C, dt)[0] == pytest.approx(4.0)


def test_score_mamba_group_form_and_einsum():
    N, M, H, G, n = 11, 6, 8, 2, 5
    B = RNG.standard_normal((N, G, n)); C = RNG.standard_normal((M, G, n))
    dt = RNG.uniform(0.1, 2, (N, H))
    s = oracle.score_mamba(B, C, dt)
    dbar = dt.reshape(N, G, H // G).mean(-1)                    # group-mean of Delta
    want = (dbar[:, None, :] * np.abs(np.einsum("ign,mgn->img", B, C))).sum((1, 2)) / (M * G)
    np.testing.assert_allclose(s, want, rtol=1e-12)
    assert (s >= 0).all()
    np.testing.assert_allclose(oracle.score_mamba(B, -3.0 * C, dt), 3.0 * s, rtol=1e-12)


def test_score_mamba_full_equals_decay_free_when_A_is_zero():
    N, M, H, G, n = 13, 4, 4, 2, 6
    B = RNG.standard_normal((N + M, G, n)); C = RNG.standard_normal((N + M, G, n))
    dt = RNG.uniform(0.1, 2, (N + M, H))
    full = oracle.score_mamba_full(B, C, dt, np.zeros(H), N)
    free = oracle.score_mamba(B[:N], C[N:], dt[:N])
    np.testing.assert_allclose(full, free, rtol=1e-13)
    decayed = oracle.score_mamba_full(B, C, dt, -np.ones(H), N)
    assert (decayed < free).all()


def test_score_mamba_full_is_impulse_response_of_the_recurrence():
    # |w_{t,j}| read off the recurrence: x = unit impulse at token j, P = 1 -> y_t = w_{t,j}
    N, M, H, G, n = 6, 3, 2, 1, 4
    T = N + M
    B = RNG.standard_normal((T, G, n)); C = RNG.standard_normal((T, G, n))
    dt = RNG.uniform(0.1, 1.5, (T, H)); A = -RNG.uniform(0.2, 1.5, H)
    want = np.zeros(N)
    for j in range(N):
        x = np.zeros((T, H, 1)); x[j] = 1.0
        y, _ = oracle.ssd_seq(x, dt, A, B, C)
        want[j] = np.abs(y[N:, :, 0]).sum() / (M * H)
    np.testing.assert_allclose(oracle.score_mamba_full(B, C, dt, A, N), want, rtol=1e-12)
    # the row-subset entry scores the listed tokens, in the listed order
    np.testing.assert_allclose(oracle.score_mamba_full(B, C, dt, A, N, rows=[4, 0, 5]), want[[4, 0, 5]], rtol=1e-12)


# ----------------------------------------------------- attention score ----

def test_score_attn_sums_to_one_and_uniform_for_zero_query():
    q = RNG.standard_normal((5, 4, 8)); k = RNG.standard_normal((33, 2, 8))
    assert oracle.score_attn(q, k).sum() == pytest.approx(1.0, rel=1e-13)
    np.testing.assert_allclose(oracle.score_attn(np.zeros_like(q), k), np.full(33, 1 / 33), rtol=1e-13)


def test_score_attn_matches_library_softmax_with_gqa():
    from scipy.special import softmax
    M, N, Hq, Hkv, d = 5, 29, 6, 2, 7
    q = RNG.standard_normal((M, Hq, d)); k = RNG.standard_normal((N, Hkv, d))
    kk = np.repeat(k, Hq // Hkv, axis=1)                         # head h reads kv head h // rep
    z = np.einsum("mhd,nhd->mhn", q, kk) * 0.37
    want = softmax(z, axis=-1).mean((0, 1))
    np.testing.assert_allclose(oracle.score_attn(q, k, scale=0.37), want, rtol=1e-12)


def test_score_attn_dominant_key_and_permutation():
    M, N, H, d = 3, 17, 2, 4
    q = np.abs(RNG.standard_normal((M, H, d))) + 0.5
    k = RNG.standard_normal((N, H, d)) * 0.01
    k[5] = 60.0
    s = oracle.score_attn(q, k)
    assert s[5] > 1 - 1e-9
    k = RNG.standard_normal((N, H, d))
    perm = RNG.permutation(N)
    np.testing.assert_allclose(oracle.score_attn(q, k[perm]), oracle.score_attn(q, k)[perm], rtol=1e-13)


# --------------------------------------------------------------- top-k ----

def test_select_topk_brute_force_tiny():
    for N in range(1, 7):
        for vals in itertools.product([0.0, 0.5, 2.0], repeat=N):
            s = np.array(vals)
            for K in range(0, N + 1):
                idx = oracle.select_topk(s, K)
                # brute force over all K-subsets: maximal score sum, then lexicographically smallest
                best = None
                for sub in itertools.combinations(range(N), K):
                    key = (-sum(s[list(sub)]), sub)
                    if best is None or key < best:
                        best = key
                assert tuple(idx) == best[1]


def test_select_topk_properties():
    s = RNG.random(500)
    idx = oracle.select_topk(s, 123)
    assert (np.diff(idx) > 0).all()
    want = np.sort(np.argsort(-s, kind="stable")[:123])
    np.testing.assert_array_equal(idx, want)
    np.testing.assert_array_equal(oracle.select_topk(s, 500), np.arange(500))
    np.testing.assert_array_equal(oracle.select_topk(np.full(40, 0.25), 9), np.arange(9))
    t = np.array([1.0, 3.0, 3.0, 0.0, 3.0, 2.0])
    np.testing.assert_array_equal(oracle.select_topk(t, 2), [1, 2])     # ties: lowest index wins
    np.testing.assert_array_equal(oracle.select_topk(t, 4), [1, 2, 4, 5])


# ------------------------------------------------------------- compact ----

def test_compact_is_row_gather_plus_text_tail():
    N, M = 20, 3
    src = RNG.integers(0, 2 ** 16, (N + M, 6)).astype(np.uint16)
    idx = np.array([0, 4, 5, 19], np.int32)
    dst, pos = oracle.compact(src, idx, N, M)
    np.testing.assert_array_equal(dst, np.concatenate([src[idx], src[N:]]))
    np.testing.assert_array_equal(pos, np.concatenate([idx, np.arange(N, N + M)]))
    dst2, pos2 = oracle.compact(src, np.arange(N, dtype=np.int32), N, M)
    np.testing.assert_array_equal(dst2, src)
    # composing two compactions composes the position maps
    idx_b = np.array([1, 3], np.int32)
    _, pos_b = oracle.compact(dst, idx_b, 4, M, pos_in=pos)
    np.testing.assert_array_equal(pos_b, [4, 19, 20, 21, 22])


# ----------------------------------------------------------- attention ----

def test_attn_matches_library_sdpa_with_gqa():
    T, Hq, Hkv, d = 23, 6, 3, 8
    q = RNG.standard_normal((T, Hq, d)); k = RNG.standard_normal((T, Hkv, d)); v = RNG.standard_normal((T, Hkv, d))
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, Hq // Hkv, 1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, Hq // Hkv, 1)).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    got = oracle.attn(q, k, v)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    rows = np.array([0, 7, 22], np.int32)
    np.testing.assert_allclose(oracle.attn(q, k, v, rows=rows), got[rows], rtol=1e-14)


def test_attn_special_cases():
    T, H, d = 9, 2, 4
    k = RNG.standard_normal((T, H, d)); v = RNG.standard_normal((T, H, d))
    o = oracle.attn(np.zeros((T, H, d)), k, v)
    want = np.cumsum(v, 0) / (np.arange(T) + 1)[:, None, None]
    np.testing.assert_allclose(o, want, rtol=1e-12)
    q = RNG.standard_normal((T, H, d))
    np.testing.assert_allclose(oracle.attn(q, k, v)[0], v[0], rtol=1e-14)   # first row sees itself only


# ------------------------------------------------------- reduced layer ----

def test_full_budget_reproduces_the_unreduced_layer():
    N, M, H, P, G, n = 40, 5, 2, 3, 1, 4
    x, dt, A, B, C, _, _ = _ssd_case(N + M, H, P, G, n, seed=77, with_D=False, with_S=False)
    s = oracle.score_mamba(B[:N], C[N:], dt[:N])
    idx = oracle.select_topk(s, N)
    xs, pos = oracle.compact(x, idx, N, M)
    np.testing.assert_array_equal(pos, np.arange(N + M))
    y_full, _ = oracle.ssd_seq(x, dt, A, B, C)
    y_red, _ = oracle.ssd_seq(xs, oracle.compact(dt, idx, N, M)[0], A, oracle.compact(B, idx, N, M)[0],
                              oracle.compact(C, idx, N, M)[0])
    np.testing.assert_array_equal(y_red, y_full)


def test_reduced_scan_runs_over_retained_positions_only():
    # dropping a token removes both its input and its decay step from the product
    N, M, H, P, G, n = 6, 2, 1, 2, 1, 3
    x, dt, A, B, C, _, _ = _ssd_case(N + M, H, P, G, n, seed=5, with_D=False, with_S=False)
    idx = np.array([0, 2, 3, 5], np.int32)
    keep = np.concatenate([idx, np.arange(N, N + M)])
    y_red, _ = oracle.ssd_seq(oracle.compact(x, idx, N, M)[0], oracle.compact(dt, idx, N, M)[0], A,
                              oracle.compact(B, idx, N, M)[0], oracle.compact(C, idx, N, M)[0])
    y_want = oracle.ssd_unrolled(x[keep], dt[keep], A, B[keep], C[keep])
    np.testing.assert_allclose(y_red, y_want, rtol=1e-12)


# ----------------------------------------------------- block glue ----------
# Pinned to library routines (torch CPU, fp64) and closed forms: the Mamba-2 block's operations
# around the scan (the paper builds on that block and does not restate them).
def test_conv1d_silu_is_a_causal_depthwise_convolution():
    import torch
    import torch.nn.functional as F
    T, C, W = 11, 6, 4
    x = RNG.standard_normal((T, C)); w = RNG.standard_normal((C, W)); b = RNG.standard_normal(C)
    t = torch.from_numpy(x.T[None])                                    # [1, C, T]
    ref = F.silu(F.conv1d(F.pad(t, (W - 1, 0)), torch.from_numpy(w[:, None, :]), torch.from_numpy(b), groups=C))
    np.testing.assert_allclose(oracle.conv1d_silu(x, w, b), ref[0].T.numpy(), rtol=1e-12, atol=1e-14)
    # causal: changing a later token leaves earlier outputs alone; token 0 sees only the last tap
    x2 = x.copy(); x2[7] += 1.0
    np.testing.assert_array_equal(oracle.conv1d_silu(x2, w, b)[:7], oracle.conv1d_silu(x, w, b)[:7])
    a0 = b + w[:, W - 1] * x[0]
    np.testing.assert_allclose(oracle.conv1d_silu(x, w, b)[0], a0 / (1 + np.exp(-a0)), rtol=1e-12)
    # width 1, unit weight, no bias: plain SiLU
    np.testing.assert_allclose(oracle.conv1d_silu(x, np.ones((C, 1))), x / (1 + np.exp(-x)), rtol=1e-12)


def test_softplus_dt_matches_library_and_limits():
    import torch
    import torch.nn.functional as F
    r = RNG.standard_normal((5, 3)) * 12; b = RNG.standard_normal(3)
    np.testing.assert_allclose(oracle.softplus_dt(r, b), np.logaddexp(0.0, r + b), rtol=1e-12)
    # torch switches to the identity above 20 (off by exp(-20) there)
    np.testing.assert_allclose(oracle.softplus_dt(r, b), F.softplus(torch.from_numpy(r + b)).numpy(), rtol=1e-8)
    big = oracle.softplus_dt(np.array([[800.0, -800.0, 0.0]]))
    assert big[0, 0] == 800.0 and big[0, 1] == 0.0 and big[0, 2] == pytest.approx(np.log(2.0))
    assert (oracle.softplus_dt(r, b) > 0).all()


def test_rmsnorm_closed_forms():
    x = RNG.standard_normal((7, 12)); w = RNG.standard_normal(12)
    np.testing.assert_allclose(oracle.rmsnorm(x, w, 1e-5), x / np.sqrt((x ** 2).mean(1, keepdims=True) + 1e-5) * w,
                               rtol=1e-12)
    out = oracle.rmsnorm(3.0 * x, np.ones(12), 0.0)                    # scale invariant, unit mean square
    np.testing.assert_allclose(out, oracle.rmsnorm(x, np.ones(12), 0.0), rtol=1e-12)
    np.testing.assert_allclose((out ** 2).mean(1), 1.0, rtol=1e-12)


def test_gated_rmsnorm_is_rmsnorm_of_the_gated_signal_per_group():
    y = RNG.standard_normal((4, 8)); z = RNG.standard_normal((4, 8)); w = RNG.standard_normal(8)
    v = y * (z / (1 + np.exp(-z)))
    one = oracle.gated_rmsnorm(y, z, w, 1, 1e-6)
    np.testing.assert_allclose(one, oracle.rmsnorm(v, w, 1e-6), rtol=1e-12)
    two = oracle.gated_rmsnorm(y, z, w, 2, 1e-6)
    for g in range(2):
        np.testing.assert_allclose(two[:, 4 * g:4 * g + 4], oracle.rmsnorm(v[:, 4 * g:4 * g + 4], w[4 * g:4 * g + 4], 1e-6),
                                   rtol=1e-12)
    # a large constant gate only scales y, which the norm (eps = 0) removes
    np.testing.assert_allclose(oracle.gated_rmsnorm(y, np.full_like(y, 50.0), w, 1, 0.0), oracle.rmsnorm(y, w, 0.0),
                               rtol=1e-9)


# ---------------------------------------------------------------- variants ----
def test_avgpool_matches_library_pooling_and_partitions_the_rows():
    N, M, D = 24, 3, 5
    src = RNG.standard_normal((N + M, D))
    for K in (24, 12, 6, 1):                                   # N % K == 0: the library's 1-D average pooling
        dst, pos = oracle.avgpool(src, N, M, K)
        ref = torch.nn.functional.avg_pool1d(torch.from_numpy(src[:N].T.copy())[None], N // K)[0].T.numpy()
        np.testing.assert_allclose(dst[:K], ref, rtol=1e-13, atol=1e-15)
        np.testing.assert_array_equal(dst[K:], src[N:])        # text tail untouched
        np.testing.assert_array_equal(pos, np.r_[np.arange(K) * (N // K), N + np.arange(M)])
    np.testing.assert_array_equal(oracle.avgpool(src, N, M, N)[0], src)   # full budget: identity
    # ragged windows (N % K != 0): sizes differ by at most one, cover every row once, keep the total
    for K in (7, 5, 23):
        dst, pos = oracle.avgpool(src, N, M, K)
        edges = np.r_[pos[:K], N]
        sizes = np.diff(edges)
        assert sizes.min() >= N // K and sizes.max() <= N // K + 1 and sizes.sum() == N
        np.testing.assert_allclose((dst[:K] * sizes[:, None]).sum(0), src[:N].sum(0), rtol=1e-12)
        for j in range(K):
            np.testing.assert_allclose(dst[j], src[edges[j]:edges[j + 1]].mean(0), rtol=1e-13, atol=1e-15)
    const = np.tile(RNG.standard_normal(D), (N + M, 1))        # a constant sequence stays constant
    np.testing.assert_allclose(oracle.avgpool(const, N, M, 7)[0], const[:7 + M], rtol=1e-14)
    p_in = np.arange(N + M, dtype=np.int32) * 3 + 2             # positions compose through pos_in
    np.testing.assert_array_equal(oracle.avgpool(src, N, M, 6, p_in)[1], np.r_[p_in[:N:4], p_in[N:]])


def test_decode_steps_continue_the_prefill():
    # scan: prefill over T tokens, then one decode step from the carried state == prefill over T + 1
    x, dt, A, B, C, D, S = _ssd_case(9, 4, 3, 2, 5, seed=5)
    y_all, S_all = oracle.ssd_seq(x, dt, A, B, C, D=D, S_in=S)
    _, S_pre = oracle.ssd_seq(x[:8], dt[:8], A, B[:8], C[:8], D=D, S_in=S)
    y1, S1 = oracle.ssd_decode_step(x[8], dt[8], A, B[8], C[8], D, S_pre)
    np.testing.assert_allclose(y1, y_all[8], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(S1, S_all, rtol=1e-12, atol=1e-13)
    # and the step itself, written out: S' = exp(dt A) S + dt x b^T, y = S' c + D x
    Hh, G = 4, 2
    for h in range(Hh):
        g = h // (Hh // G)
        Sn = np.exp(dt[8, h] * A[h]) * S_pre[h] + dt[8, h] * np.outer(x[8, h], B[8, g])
        np.testing.assert_allclose(S1[h], Sn, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(y1[h], Sn @ C[8, g] + D[h] * x[8, h], rtol=1e-12, atol=1e-13)
    # attention: the new token against the whole cache == library softmax attention of one query
    T, Hq, Hkv, d = 11, 4, 2, 6
    q1 = RNG.standard_normal((Hq, d)); k = RNG.standard_normal((T, Hkv, d)); v = RNG.standard_normal((T, Hkv, d))
    o = oracle.attn_decode_step(q1, k, v)
    kk = torch.from_numpy(k).repeat_interleave(Hq // Hkv, 1).permute(1, 0, 2)
    vv = torch.from_numpy(v).repeat_interleave(Hq // Hkv, 1).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q1)[:, None], kk, vv)[:, 0].numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------ reference blocks -------
def _library_mamba_block(hidden, N, M, wt, H, P, G, n, idx, eps):
    """The published Mamba-2 block put together from torch's own routines (fp64), the scan as the
    plain token-by-token recurrence; idx (kept vision tokens) is applied after the convolution."""
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    h = t(hidden)
    d_inner, gn = H * P, G * n
    u = F.rms_norm(h, (h.shape[1],), t(wt["norm_w"]), eps)
    z = u @ t(wt["W_z"])
    xbcdt = u @ t(wt["W_xbcdt"])
    C_all = d_inner + 2 * gn
    W = wt["conv_w"].shape[1]
    conv = F.conv1d(xbcdt[:, :C_all].T[None], t(wt["conv_w"])[:, None, :], t(wt["conv_b"]), padding=W - 1,
                    groups=C_all)[0, :, : h.shape[0]].T
    xbc = F.silu(conv)
    dt = F.softplus(xbcdt[:, C_all:] + t(wt["dt_bias"]))
    if idx is not None:
        keep = torch.cat([torch.from_numpy(np.asarray(idx)).long(), torch.arange(N, N + M)])
        xbc, dt, z, h = xbc[keep], dt[keep], z[keep], h[keep]
    T = xbc.shape[0]
    x = xbc[:, :d_inner].reshape(T, H, P)
    B = xbc[:, d_inner:d_inner + gn].reshape(T, G, n).repeat_interleave(H // G, 1)
    C = xbc[:, d_inner + gn:].reshape(T, G, n).repeat_interleave(H // G, 1)
    A, D = t(wt["A"]), t(wt["D"])
    S = torch.zeros(H, P, n, dtype=torch.float64)
    y = torch.empty(T, H, P, dtype=torch.float64)
    for i in range(T):
        S = torch.exp(dt[i] * A)[:, None, None] * S + dt[i][:, None, None] * x[i][:, :, None] * B[i][:, None, :]
        y[i] = torch.einsum("hpn,hn->hp", S, C[i]) + D[:, None] * x[i]
    v = (y.reshape(T, d_inner) * F.silu(z)).reshape(T, G, d_inner // G)
    g = (F.rms_norm(v, (d_inner // G,), None, eps).reshape(T, d_inner)) * t(wt["gnorm_w"])
    return (g @ t(wt["W_out"]) + h).numpy()


def _library_attn_block(hidden, N, M, wt, Hq, Hkv, d, idx, eps):
    F = torch.nn.functional
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    h = t(hidden)
    u = F.rms_norm(h, (h.shape[1],), t(wt["norm_w"]), eps)
    q, k, v = u @ t(wt["W_q"]), u @ t(wt["W_k"]), u @ t(wt["W_v"])
    if idx is not None:
        keep = torch.cat([torch.from_numpy(np.asarray(idx)).long(), torch.arange(N, N + M)])
        q, k, v, h = q[keep], k[keep], v[keep], h[keep]
    T = q.shape[0]
    q = q.reshape(T, Hq, d).permute(1, 0, 2)
    k = k.reshape(T, Hkv, d).repeat_interleave(Hq // Hkv, 1).permute(1, 0, 2)
    v = v.reshape(T, Hkv, d).repeat_interleave(Hq // Hkv, 1).permute(1, 0, 2)
    o = F.scaled_dot_product_attention(q, k, v, is_causal=True).permute(1, 0, 2).reshape(T, Hq * d)
    return (o @ t(wt["W_o"]) + h).numpy()


@pytest.mark.parametrize("reduced", [False, True])
def test_reference_blocks_match_a_composition_of_library_routines(reduced):
    """The reference blocks (which chain the oracle's routines) against the same blocks assembled from
    torch's rms_norm, grouped conv1d, silu, softplus and scaled_dot_product_attention.  The reference
    rounds every stored tensor to the device's type; with "f32" that rounding is far below the
    tolerance, so this pins the order of the stages, the x | B | C | dt split, the gate, the grouped
    norm, the residual and what is compacted."""
    import oracle.blocks as ref
    rng = np.random.default_rng(11)
    N, M, dm, H, P, G, n, W = 40, 6, 24, 4, 8, 2, 6, 4
    d_inner, gn = H * P, G * n
    wt = {"norm_w": 1 + 0.1 * rng.standard_normal(dm), "W_z": rng.standard_normal((dm, d_inner)) / dm ** 0.5,
          "W_xbcdt": rng.standard_normal((dm, d_inner + 2 * gn + H)) / dm ** 0.5,
          "conv_w": rng.standard_normal((d_inner + 2 * gn, W)) / 2, "conv_b": 0.1 * rng.standard_normal(d_inner + 2 * gn),
          "dt_bias": rng.standard_normal(H) - 1, "A": -np.exp(rng.standard_normal(H)), "D": rng.standard_normal(H),
          "gnorm_w": 1 + 0.1 * rng.standard_normal(d_inner), "W_out": rng.standard_normal((d_inner, dm)) / d_inner ** 0.5}
    hidden = rng.standard_normal((N + M, dm))
    idx = np.sort(rng.choice(N, 13, replace=False)).astype(np.int32) if reduced else None
    got, _ = ref.mamba_block(hidden, N, M, wt, H, P, G, n, "f32", idx=idx, eps=1e-5)
    want = _library_mamba_block(hidden, N, M, wt, H, P, G, n, idx, 1e-5)
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=2e-5)

    Hq, Hkv, d = 4, 2, 8
    wa = {"norm_w": 1 + 0.1 * rng.standard_normal(dm), "W_q": rng.standard_normal((dm, Hq * d)) / dm ** 0.5,
          "W_k": rng.standard_normal((dm, Hkv * d)) / dm ** 0.5, "W_v": rng.standard_normal((dm, Hkv * d)) / dm ** 0.5,
          "W_o": rng.standard_normal((Hq * d, dm)) / (Hq * d) ** 0.5}
    got, _ = ref.attn_block(hidden, N, M, wa, Hq, Hkv, d, "f32", idx=idx, eps=1e-5)
    want = _library_attn_block(hidden, N, M, wa, Hq, Hkv, d, idx, 1e-5)
    np.testing.assert_allclose(got, want, rtol=2e-5, atol=2e-5)
