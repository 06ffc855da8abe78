"""Parity at the benchmark's full sizes, in the launch configuration bench.py times: whatever the
fp64 oracle can afford is compared in full (scores, indices, gathers), the mixers on sampled
heads / query rows computed one by one, plus properties that hold at any size.  Needs a GPU."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_00198_amd as strd
from paper_2603_00198_amd import synth
from util import TOL, assert_close, assert_topk_equivalent

pytestmark = pytest.mark.gpu
DEV = "cuda"
f = synth.np64
TOLB = TOL[torch.bfloat16]


def _say(msg):
    print("[case] " + msg, flush=True)


def _reduced_mamba(w, t, hidden):
    N, M, K = w.N, w.M, w.K
    s = strd.score_mamba(t["B"][:N].contiguous(), t["C"][N:].contiguous(), t["dt"][:N].contiguous())
    idx = strd.select_topk(s, K)
    keys = ("x", "B", "C", "dt")
    outs, pos = strd.compact_batch([t[k] for k in keys] + [hidden], idx, N, M, want_pos=True)
    red = dict(zip(keys + ("hidden",), outs))
    y, S = strd.ssd_prefill(red["x"], red["dt"], t["A"], red["B"], red["C"], chunk=w.mamba.chunk)
    return s, idx, pos, red, y, S


def _check_ssd_heads(x, dt, A, B, C, y, S, heads, G, what):
    """Oracle recurrence for a few heads at full length."""
    H = x.shape[1]
    hpg = H // G
    for h in heads:
        g = h // hpg
        y_ref, S_ref = oracle.ssd_seq(f(x[:, h:h + 1]), f(dt[:, h:h + 1]), f(A[h:h + 1]), f(B[:, g:g + 1]),
                                      f(C[:, g:g + 1]))
        assert_close(f(y[:, h:h + 1]), y_ref, TOLB, "%s y head %d" % (what, h), units=(1,))
        if S is not None:
            assert_close(f(S[h:h + 1]), S_ref, TOLB, "%s state head %d" % (what, h), units=(0,))


def test_c2_reduced_mamba_layer_full_size():
    w = synth.WORKLOADS["c2"]
    _say("c2 full size: N=%d M=%d K=%d" % (w.N, w.M, w.K))
    hidden = synth.hidden_states(w, DEV)
    t = synth.mamba_inputs(w, hidden)
    hb = hidden.to(torch.bfloat16)
    N, M, K = w.N, w.M, w.K
    s, idx, pos, red, y, S = _reduced_mamba(w, t, hb)
    s_ref = oracle.score_mamba(f(t["B"][:N]), f(t["C"][N:]), f(t["dt"][:N]))
    assert_close(s.cpu().numpy(), s_ref, TOLB, "scores", units=(0,))
    swaps = assert_topk_equivalent(idx.cpu().numpy(), s_ref, K, TOLB)
    _say("near-tie swaps vs oracle: %d of %d" % (swaps, K))
    # select on the oracle's exact scores (rounded to fp32) is bit-exact
    s32 = torch.from_numpy(s_ref.astype(np.float32)).to(DEV)
    np.testing.assert_array_equal(strd.select_topk(s32, K).cpu().numpy(),
                                  oracle.select_topk(s_ref.astype(np.float32).astype(np.float64), K))
    i_np = idx.cpu().numpy()
    for k in ("x", "B", "C", "hidden"):
        src = (hb if k == "hidden" else t[k]).view(torch.int16).cpu().numpy()
        np.testing.assert_array_equal(red[k].view(torch.int16).cpu().numpy(), oracle.compact(src, i_np, N, M)[0])
    np.testing.assert_array_equal(red["dt"].cpu().numpy(), oracle.compact(t["dt"].cpu().numpy(), i_np, N, M)[0])
    np.testing.assert_array_equal(pos.cpu().numpy(), np.concatenate([i_np, np.arange(N, N + M)]))
    heads = [0, 17, 34, 51, 68, 85, 102, 127]       # one per group
    _check_ssd_heads(red["x"], red["dt"], t["A"], red["B"], red["C"], y, S, heads, w.mamba.G, "reduced")
    # the scan that gathers its inputs through idx gives the same bits without the compacted copies
    y_g, S_g = strd.ssd_prefill_gather(t["x"], t["dt"], t["A"], t["B"], t["C"], idx, N, M, chunk=w.mamba.chunk)
    assert torch.equal(y_g, y) and torch.equal(S_g, S)
    # the unreduced layer (the denominator of the speed-up) on two heads
    y_full, S_full = strd.ssd_prefill(t["x"], t["dt"], t["A"], t["B"], t["C"], chunk=w.mamba.chunk)
    _check_ssd_heads(t["x"], t["dt"], t["A"], t["B"], t["C"], y_full, S_full, [5, 120], w.mamba.G, "full")
    assert torch.isfinite(y_full.float()).all()


def test_c3_reduced_attention_layer_full_size():
    w = synth.WORKLOADS["c3"]
    _say("c3 full size: N=%d M=%d K=%d" % (w.N, w.M, w.K))
    hidden = synth.hidden_states(w, DEV)
    t = synth.attn_inputs(w, hidden)
    N, M, K = w.N, w.M, w.K
    s = strd.score_attn(t["q"][N:].contiguous(), t["k"][:N].contiguous())
    idx = strd.select_topk(s, K)
    (qs, ks, vs), _ = strd.compact_batch([t["q"], t["k"], t["v"]], idx, N, M)
    o = strd.attn_prefill(qs, ks, vs)
    assert abs(float(s.double().sum()) - 1.0) < 1e-3 and float(s.min()) >= 0.0
    _say("oracle scores (about 70 G multiply-adds in fp64) ...")
    s_ref = oracle.score_attn(f(t["q"][N:]), f(t["k"][:N]))
    assert_close(s.cpu().numpy(), s_ref, TOLB, "scores", units=(0,))
    swaps = assert_topk_equivalent(idx.cpu().numpy(), s_ref, K, TOLB)
    _say("near-tie swaps vs oracle: %d of %d" % (swaps, K))
    i_np = idx.cpu().numpy()
    np.testing.assert_array_equal(ks.view(torch.int16).cpu().numpy(),
                                  oracle.compact(t["k"].view(torch.int16).cpu().numpy(), i_np, N, M)[0])
    Tr = K + M
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 63, 64, 127, 128, 129, Tr - 1, Tr - 2, K - 1, K, K + 1],
                                     np.random.default_rng(0).integers(0, Tr, 10)])).astype(np.int32)
    o_ref = oracle.attn(f(qs), f(ks), f(vs), rows=rows)
    assert_close(f(o[torch.from_numpy(rows).long().to(DEV)]), o_ref, TOLB, "reduced attention rows", units=(0, 1))
    # the unreduced layer on a few rows
    o_full = strd.attn_prefill(t["q"], t["k"], t["v"])
    rows = np.array([0, 200, 4095, 4096, 20000, N + M - 1], np.int32)
    o_ref = oracle.attn(f(t["q"]), f(t["k"]), f(t["v"]), rows=rows)
    assert_close(f(o_full[torch.from_numpy(rows).long().to(DEV)]), o_ref, TOLB, "full attention rows", units=(0, 1))


@pytest.mark.parametrize("a_scale", [1.0, 3e-4])
def test_c2_full_dynamic_score_sampled(a_scale):
    """The decayed score at c2 size on sampled tokens (each token's score is independent).  With the
    workload's A only the last tokens are above fp32's range; A x 3e-4 keeps the whole sequence alive."""
    w = synth.WORKLOADS["c2"]
    _say("c2 full dynamic score: N=%d M=%d, A x %g" % (w.N, w.M, a_scale))
    hidden = synth.hidden_states(w, DEV)
    t = synth.mamba_inputs(w, hidden)
    N = w.N
    A = (t["A"] * a_scale).contiguous()
    s = strd.score_mamba_full(t["B"][:N].contiguous(), t["C"][N:].contiguous(), t["dt"], A)
    rng = np.random.default_rng(2)
    pick = np.unique(np.concatenate([np.arange(N - 12, N), rng.choice(N - 12, 20, replace=False)])).astype(np.int32)
    want = oracle.score_mamba_full(f(t["B"]), f(t["C"]), f(t["dt"]), f(A), N, rows=pick)
    got = s.cpu().numpy()[pick]
    assert np.isfinite(s.cpu().numpy()).all() and (s.cpu().numpy() >= 0).all()
    # relative to the largest score of the sample (which contains the last tokens, the largest of all)
    assert np.abs(got - want).max() <= TOLB * want.max()
    if a_scale < 1:
        assert (want > 1e-3 * want.max()).all()     # the sample is not vacuous: early tokens still count
        assert (np.abs(got - want) <= TOLB * want).all()


@pytest.mark.parametrize("budget", [0.10, 0.25, 0.50])
def test_c5_long_video_mamba_layer_sampled(budget):
    w = synth.shrink(synth.WORKLOADS["c5"], N=131072, M=512, budget=budget)
    _say("c5 long video mamba: N=%d M=%d K=%d" % (w.N, w.M, w.K))
    hidden = synth.hidden_states(w, DEV)
    t = synth.mamba_inputs(w, hidden)
    hb = hidden.to(torch.bfloat16)
    del hidden
    N, M, K = w.N, w.M, w.K
    s, idx, pos, red, y, S = _reduced_mamba(w, t, hb)
    # scores of sampled tokens, one by one (a token's score needs only its own row)
    pick = np.sort(np.random.default_rng(1).choice(N, 192, replace=False))
    pt = torch.from_numpy(pick).long().to(DEV)
    s_ref = oracle.score_mamba(f(t["B"][:N][pt]), f(t["C"][N:]), f(t["dt"][:N][pt]))
    assert_close(s[pt].cpu().numpy(), s_ref, TOLB, "sampled scores", units=(0,))
    # selection: valid, ascending, consistent with a threshold on the device scores
    i_np = idx.cpu().numpy()
    s_np = s.cpu().numpy()
    assert i_np.shape == (K,) and (np.diff(i_np) > 0).all() and i_np[0] >= 0 and i_np[-1] < N
    np.testing.assert_array_equal(i_np, oracle.select_topk(s_np.astype(np.float64), K))
    np.testing.assert_array_equal(red["B"].view(torch.int16).cpu().numpy(),
                                  oracle.compact(t["B"].view(torch.int16).cpu().numpy(), i_np, N, M)[0])
    np.testing.assert_array_equal(red["hidden"][::97].view(torch.int16).cpu().numpy(),
                                  hb[torch.from_numpy(np.concatenate([i_np, np.arange(N, N + M)])[::97]).long().to(DEV)]
                                  .view(torch.int16).cpu().numpy())
    _check_ssd_heads(red["x"], red["dt"], t["A"], red["B"], red["C"], y, S, [3, 77], w.mamba.G, "reduced")
    y_g, S_g = strd.ssd_prefill_gather(t["x"], t["dt"], t["A"], t["B"], t["C"], idx, N, M, chunk=w.mamba.chunk)
    assert torch.equal(y_g, y) and torch.equal(S_g, S)


@pytest.mark.parametrize("budget", [0.10, 0.25, 0.50])
def test_c5_long_video_attention_layer_sampled(budget):
    w = synth.shrink(synth.WORKLOADS["c5"], N=131072, M=512, budget=budget)
    _say("c5 long video attention: N=%d M=%d K=%d" % (w.N, w.M, w.K))
    hidden = synth.hidden_states(w, DEV)
    t = synth.attn_inputs(w, hidden)
    del hidden
    N, M, K = w.N, w.M, w.K
    q_txt, k_vis = t["q"][N:].contiguous(), t["k"][:N].contiguous()
    s = strd.score_attn(q_txt, k_vis)
    # properties that hold at any size: a probability vector; independent of the key order
    assert abs(float(s.double().sum()) - 1.0) < 1e-3 and float(s.min()) >= 0.0
    # exact values on a key subset whose softmax normaliser the oracle can afford: restrict both sides to 2048 keys
    sub = torch.from_numpy(np.sort(np.random.default_rng(2).choice(N, 2048, replace=False))).long().to(DEV)
    s_sub = strd.score_attn(q_txt, k_vis[sub].contiguous())
    assert_close(s_sub.cpu().numpy(), oracle.score_attn(f(q_txt), f(k_vis[sub])), TOLB, "subset scores", units=(0,))
    if budget == 0.25:
        # ... and over all 131072 keys for a subset of the text rows (a row's softmax is independent of the others)
        _say("oracle scores of 21 text rows over all keys ...")
        q_few = q_txt[::25].contiguous()
        s_few = strd.score_attn(q_few, k_vis)
        assert_close(s_few.cpu().numpy(), oracle.score_attn(f(q_few), f(k_vis)), TOLB, "scores of a text-row subset",
                     units=(0,))
    idx = strd.select_topk(s, K)
    i_np = idx.cpu().numpy()
    np.testing.assert_array_equal(i_np, oracle.select_topk(s.cpu().numpy().astype(np.float64), K))
    (qs, ks, vs), _ = strd.compact_batch([t["q"], t["k"], t["v"]], idx, N, M)
    np.testing.assert_array_equal(vs[::61].view(torch.int16).cpu().numpy(),
                                  t["v"][torch.from_numpy(np.concatenate([i_np, np.arange(N, N + M)])[::61]).long().to(DEV)]
                                  .view(torch.int16).cpu().numpy())
    o = strd.attn_prefill(qs, ks, vs)
    Tr = K + M
    rows = np.array([0, 127, 128, 5000, K - 1, K, Tr - 1], np.int32)
    o_ref = oracle.attn(f(qs), f(ks), f(vs), rows=rows)
    assert_close(f(o[torch.from_numpy(rows).long().to(DEV)]), o_ref, TOLB, "reduced attention rows", units=(0, 1))


def test_variants_at_benchmark_shapes():
    """Average-pool baseline on the c2 residual stream and one decode token at the c2 state / the c3
    reduced cache: the shapes `bench.py` times under `next_rows.variants`, compared in full."""
    _say("variants at c2 / c3 shapes")
    wm, wa = synth.WORKLOADS["c2"], synth.WORKLOADS["c3"]
    g = torch.Generator(device=DEV).manual_seed(11)
    hid = torch.randn(wm.T, wm.d_model, generator=g, device=DEV).to(torch.bfloat16)
    dst, pos = strd.avgpool(hid, wm.N, wm.M, wm.K, want_pos=True)
    want, want_pos = oracle.avgpool(f(hid), wm.N, wm.M, wm.K)
    np.testing.assert_array_equal(pos.cpu().numpy(), want_pos)
    assert_close(f(dst), want, TOLB, "avgpool c2")

    m = wm.mamba
    x = torch.randn(m.H, m.P, generator=g, device=DEV).to(torch.bfloat16)
    B = torch.randn(m.G, m.n, generator=g, device=DEV).to(torch.bfloat16)
    C = torch.randn(m.G, m.n, generator=g, device=DEV).to(torch.bfloat16)
    dt = torch.rand(m.H, generator=g, device=DEV) + 0.05
    A = -torch.exp(2 * torch.rand(m.H, generator=g, device=DEV))
    S = torch.randn(m.H, m.P, m.n, generator=g, device=DEV)
    S0 = f(S)
    y = strd.ssd_decode_step(x, dt, A, B, C, None, S)
    y_ref, S_ref = oracle.ssd_decode_step(f(x), f(dt), f(A), f(B), f(C), None, S0)
    assert_close(f(S), S_ref, 1e-5, "decode state c2")
    assert_close(f(y), y_ref, TOLB, "decode y c2", units=(0,))

    a = wa.attn
    T = wa.K + wa.M + 1
    q = torch.randn(a.Hq, a.d, generator=g, device=DEV).to(torch.bfloat16)
    kc = torch.randn(T, a.Hkv, a.d, generator=g, device=DEV).to(torch.bfloat16)
    vc = torch.randn(T, a.Hkv, a.d, generator=g, device=DEV).to(torch.bfloat16)
    o = strd.attn_decode_step(q, kc, vc)
    assert_close(f(o), oracle.attn_decode_step(f(q), f(kc), f(vc)), TOLB, "attn decode c3 reduced cache", units=(0,))


def test_c4_block_projections_sampled():
    """The projections of a c4 block at their full size (33 024 tokens; 4096 -> 18 560 in, 8192 -> 4096 out with the
    residual), as `bench.py --block-stack` launches them: the library's own kernel through strd_linear.  Sampled
    elements, the edges of the output and whole rows against the dense product in fp64; the same call by rocBLAS
    within the same tolerance."""
    w = synth.WORKLOADS["c4"]
    T = w.T
    g = torch.Generator(device="cpu").manual_seed(7)
    rng = np.random.default_rng(7)
    for Kd, Nd, with_res in ((w.d_model, 18560, False), (2 * w.d_model, w.d_model, True)):
        _say("c4 projection: T=%d Kd=%d Nd=%d residual=%s" % (T, Kd, Nd, with_res))
        assert strd.linear_mfma_supported(T, Kd, Nd, torch.bfloat16)
        x = torch.randn(T, Kd, generator=g).to(torch.bfloat16).to(DEV)
        wt = (torch.randn(Kd, Nd, generator=g) / Kd ** 0.5).to(torch.bfloat16).to(DEV)
        r = torch.randn(T, Nd, generator=g).to(torch.bfloat16).to(DEV) if with_res else None
        out = strd.linear(x, wt, r)
        assert torch.equal(out, strd.linear_mfma(x, wt, r))            # the size picks the library's own kernel
        ts = np.concatenate([rng.integers(0, T, 400), [0, 255, 256, T - 257, T - 256, T - 1]])
        ns = np.concatenate([rng.integers(0, Nd, 400), [0, 255, 256, Nd - 257, Nd - 9, Nd - 1]])
        ti, ni = torch.from_numpy(ts).long().to(DEV), torch.from_numpy(ns).long().to(DEV)
        want = f(x[ti]) @ f(wt[:, ni])                                  # [406, 406]: every sampled row x every sampled column
        if with_res:
            want = want + f(r[ti][:, ni])
        assert_close(f(out[ti][:, ni]), want, TOLB, "sampled block")
        whole = f(x[ti[-3:]]) @ f(wt) + (f(r[ti[-3:]]) if with_res else 0.0)
        assert_close(f(out[ti[-3:]]), whole, TOLB, "whole rows")
        assert_close(f(strd.linear_library(x, wt, r)[ti][:, ni]), want, TOLB, "the same by the library product")
        del x, wt, r, out
