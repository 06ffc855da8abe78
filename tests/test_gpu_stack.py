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
            assert_close(got[l]["scores"].cpu().numpy(), s_ref, tol, "layer %d scores" % l)
            idx = got[l]["idx"].cpu().numpy()
            assert_topk_equivalent(idx, s_ref, K, tol)
            # continue the chain on the device's own selection (near-ties may legitimately differ)
            cur = {k: oracle.compact(v, idx, n_cur, M)[0] for k, v in cur.items()}
            pos = oracle.compact(pos.reshape(-1, 1), idx, n_cur, M)[0].reshape(-1)
            n_cur = K
        np.testing.assert_array_equal(got[l]["pos"].cpu().numpy(), pos)
        if kind == "mamba":
            y_ref, S_ref = oracle.ssd_seq(cur["x"], cur["dt"], t["A"], cur["B"], cur["C"])
            assert_close(f(got[l]["y"]), y_ref, tol, "layer %d y" % l)
            assert_close(f(got[l]["state"]), S_ref, tol, "layer %d state" % l)
        else:
            assert_close(f(got[l]["y"]), oracle.attn(cur["q"], cur["k"], cur["v"]), tol, "layer %d o" % l)
        assert got[l]["y"].shape[0] == budgets[l] + M
