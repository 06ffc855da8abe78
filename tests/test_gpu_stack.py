"""The 8-layer progressive stack (6 Mamba-2 + 2 attention layers, retention 100/100/75/75/50/50/25/25 %)
on a shortened sequence, against the same chain evaluated with the CPU oracle.  Needs a GPU."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_00198_amd as strd
from paper_2603_00198_amd import stack, synth
from util import TOL, assert_close, assert_topk_equivalent

pytestmark = pytest.mark.gpu


def test_progressive_stack_matches_oracle_chain():
    w = synth.shrink(synth.WORKLOADS["c4"], N=2048, M=48, d_model=256,
                     mamba=synth.MambaShape(H=16, P=64, n=128, G=2, chunk=256), attn=synth.AttnShape(Hq=8, Hkv=2, d=128))
    print("[case] stack N=%d M=%d" % (w.N, w.M), flush=True)
    N, M = w.N, w.M
    kinds = synth.C4_LAYERS
    budgets = strd.schedule_budgets(list(synth.C4_RETAIN), N)
    assert budgets == [2048, 2048, 1536, 1536, 1024, 1024, 512, 512]
    hidden = synth.hidden_states(w, "cuda")
    layers = []
    for l, kind in enumerate(kinds):
        h_l = synth.hidden_states(w, "cuda", seed=100 + l)
        layers.append(synth.mamba_inputs(w, h_l, seed=l) if kind == "mamba" else synth.attn_inputs(w, h_l, seed=l))
    got = stack.run_stack(kinds, layers, hidden.to(torch.bfloat16), N, M, budgets)

    f = synth.np64
    tol = TOL[torch.bfloat16]
    pos = np.arange(N + M, dtype=np.int32)
    n_cur = N
    for l, kind in enumerate(kinds):
        t = {k: f(v) for k, v in layers[l].items()}
        keys = ("x", "B", "C", "dt") if kind == "mamba" else ("q", "k", "v")
        cur = {k: t[k][pos] for k in keys}
        K = budgets[l]
        if K < n_cur:
            if kind == "mamba":
                s_ref = oracle.score_mamba(cur["B"][:n_cur], cur["C"][n_cur:], cur["dt"][:n_cur])
            else:
                s_ref = oracle.score_attn(cur["q"][n_cur:], cur["k"][:n_cur])
            assert_close(got[l]["scores"].cpu().numpy(), s_ref, tol, "layer %d scores" % l, units=(0,))
            idx = got[l]["idx"].cpu().numpy()
            assert_topk_equivalent(idx, s_ref, K, tol)
            # continue the chain on the device's own selection (near-ties may legitimately differ)
            cur = {k: oracle.compact(v, idx, n_cur, M)[0] for k, v in cur.items()}
            pos = oracle.compact(pos.reshape(-1, 1), idx, n_cur, M)[0].reshape(-1)
            n_cur = K
        np.testing.assert_array_equal(got[l]["pos"].cpu().numpy(), pos)
        if kind == "mamba":
            y_ref, S_ref = oracle.ssd_seq(cur["x"], cur["dt"], t["A"], cur["B"], cur["C"])
            assert_close(f(got[l]["y"]), y_ref, tol, "layer %d y" % l, units=(1,))
            assert_close(f(got[l]["state"]), S_ref, tol, "layer %d state" % l, units=(0,))
        else:
            assert_close(f(got[l]["y"]), oracle.attn(cur["q"], cur["k"], cur["v"]), tol, "layer %d o" % l, units=(0, 1))
        assert got[l]["y"].shape[0] == budgets[l] + M


def test_progressive_stack_at_full_size_sampled():
    """The same stack at the size of the workload (32768 vision + 256 text tokens, the layer shapes
    of the single-layer workloads): scores and position maps of every reducing layer in full, the
    selection bit-exact on the device's own scores and equivalent to the oracle's, the mixers on
    sampled heads / query rows computed one by one by the oracle."""
    w = synth.WORKLOADS["c4"]
    N, M = w.N, w.M
    print("[case] full-size stack N=%d M=%d" % (N, M), flush=True)
    kinds = synth.C4_LAYERS
    budgets = strd.schedule_budgets(list(synth.C4_RETAIN), N)
    assert budgets == [32768, 32768, 24576, 24576, 16384, 16384, 8192, 8192]
    hidden = synth.hidden_states(w, "cuda").to(torch.bfloat16)
    layers = []
    for l, kind in enumerate(kinds):
        h_l = synth.hidden_states(w, "cuda", seed=100 + l)
        layers.append(synth.mamba_inputs(w, h_l, seed=l) if kind == "mamba" else synth.attn_inputs(w, h_l, seed=l))
        del h_l
    got = stack.run_stack(kinds, layers, hidden, N, M, budgets)
    torch.cuda.synchronize()

    f = synth.np64
    tol = TOL[torch.bfloat16]
    pos = np.arange(N + M, dtype=np.int32)
    n_cur = N
    reduced_kinds = []
    hpg = w.mamba.H // w.mamba.G
    for l, kind in enumerate(kinds):
        print("[case]   layer %d (%s), %d vision tokens in" % (l, kind, n_cur), flush=True)
        t = layers[l]
        rows_dev = torch.from_numpy(pos).long().cuda()
        K = budgets[l]
        if K < n_cur:
            vis, txt = rows_dev[:n_cur], rows_dev[n_cur:]
            if kind == "mamba":
                s_ref = oracle.score_mamba(f(t["B"][vis]), f(t["C"][txt]), f(t["dt"][vis]))
            else:
                s_ref = oracle.score_attn(f(t["q"][txt]), f(t["k"][vis]))
            s_dev = got[l]["scores"].cpu().numpy()
            assert_close(s_dev, s_ref, tol, "layer %d scores" % l, units=(0,))
            idx = got[l]["idx"].cpu().numpy()
            np.testing.assert_array_equal(idx, oracle.select_topk(s_dev.astype(np.float64), K))
            assert_topk_equivalent(idx, s_ref, K, tol)
            pos = np.concatenate([pos[:n_cur][idx], pos[n_cur:]])
            rows_dev = torch.from_numpy(pos).long().cuda()
            n_cur = K
            reduced_kinds.append(kind)
        np.testing.assert_array_equal(got[l]["pos"].cpu().numpy(), pos)
        assert got[l]["y"].shape[0] == budgets[l] + M
        if kind == "mamba":
            for h in (3 + 7 * l, 127 - 11 * l):
                g = h // hpg
                y_ref, S_ref = oracle.ssd_seq(f(t["x"][rows_dev, h:h + 1]), f(t["dt"][rows_dev, h:h + 1]), f(t["A"][h:h + 1]),
                                              f(t["B"][rows_dev, g:g + 1]), f(t["C"][rows_dev, g:g + 1]))
                assert_close(f(got[l]["y"][:, h:h + 1]), y_ref, tol, "layer %d y head %d" % (l, h), units=(1,))
                assert_close(f(got[l]["state"][h:h + 1]), S_ref, tol, "layer %d state head %d" % (l, h), units=(0,))
        else:
            Tr = n_cur + M
            rows = np.array([0, 1, 255, 256, 4099, n_cur - 1, n_cur, Tr - 1], np.int32)
            o_ref = oracle.attn(f(t["q"][rows_dev]), f(t["k"][rows_dev]), f(t["v"][rows_dev]), rows=rows)
            assert_close(f(got[l]["y"][torch.from_numpy(rows).long().cuda()]), o_ref, tol, "layer %d o rows" % l, units=(0, 1))
    assert sorted(reduced_kinds) == ["attn", "mamba", "mamba"]     # both scores were used inside the stack
