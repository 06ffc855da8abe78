"""Hidden-to-hidden blocks (projections, Mamba-2 / attention glue, mixer, residual) with token
reduction inside, against the reference blocks built from the fp64 oracle.  Needs a GPU."""
import numpy as np
import pytest
import torch

import oracle
import oracle.blocks as ref
import paper_2603_00198_amd as strd
from paper_2603_00198_amd import blocks, synth
from util import TOL, assert_close, assert_topk_equivalent

pytestmark = pytest.mark.gpu
DEV = "cuda"
f = synth.np64

W = synth.Workload("blocks", N=300, M=20, d_model=256, dtype="bf16",
                   mamba=synth.MambaShape(H=8, P=32, n=64, G=2, chunk=64), attn=synth.AttnShape(Hq=4, Hkv=2, d=64))
TOLB = TOL[torch.bfloat16]


def _say(msg):
    print("[case] " + msg, flush=True)


def _np(wt):
    return {k: f(v) for k, v in wt.items()}


@pytest.mark.parametrize("K", [None, 75, 1])
def test_mamba_block_matches_reference(K):
    _say("mamba block N=%d M=%d K=%s" % (W.N, W.M, K))
    s = W.mamba
    hidden = synth.hidden_states(W, DEV).to(torch.bfloat16)
    wt = synth.mamba_block_weights(W, DEV)
    out, n_left, info = blocks.mamba_block(hidden, W.N, W.M, wt, s, K)
    idx = info["idx"].cpu().numpy() if info else None
    want, pre = ref.mamba_block(f(hidden), W.N, W.M, _np(wt), s.H, s.P, s.G, s.n, "bf16", idx)
    assert n_left == (K if K else W.N) and out.shape == (n_left + W.M, W.d_model)
    assert_close(f(out), want, TOLB, "mamba block output")
    if info:   # the block scored with its own post-convolution b, c and post-softplus dt
        s_ref = oracle.score_mamba(pre["B"][:W.N], pre["C"][W.N:], pre["dt"][:W.N])
        assert_close(info["scores"].cpu().numpy(), s_ref, TOLB, "block scores", units=(0,))
        assert_topk_equivalent(idx, s_ref, K, TOLB)


@pytest.mark.parametrize("K", [None, 150])
def test_attention_block_matches_reference(K):
    _say("attention block N=%d M=%d K=%s" % (W.N, W.M, K))
    s = W.attn
    hidden = synth.hidden_states(W, DEV).to(torch.bfloat16)
    wt = synth.attn_block_weights(W, DEV)
    out, n_left, info = blocks.attn_block(hidden, W.N, W.M, wt, s, K)
    idx = info["idx"].cpu().numpy() if info else None
    want, pre = ref.attn_block(f(hidden), W.N, W.M, _np(wt), s.Hq, s.Hkv, s.d, "bf16", idx)
    assert_close(f(out), want, TOLB, "attention block output")
    if info:
        s_ref = oracle.score_attn(pre["q"][W.N:], pre["k"][:W.N])
        assert_close(info["scores"].cpu().numpy(), s_ref, TOLB, "block scores", units=(0,))
        assert_topk_equivalent(idx, s_ref, K, TOLB)


def test_three_block_stack_with_progressive_budgets():
    """A stack of blocks with reduction inside.  Every block is checked at the plain tolerance against
    the reference block applied to what the device handed to it (the device's own bf16 hidden states
    and the device's own selection), so rounding does not compound from block to block; the stack
    driver must return exactly what the blocks return one after the other."""
    kinds = ("mamba", "attn", "mamba")
    budgets = strd.schedule_budgets([1.0, 0.5, 0.25], W.N)
    _say("block stack %s budgets %s" % (kinds, budgets))
    hidden = synth.hidden_states(W, DEV).to(torch.bfloat16)
    wts = [synth.mamba_block_weights(W, DEV, 0), synth.attn_block_weights(W, DEV, 1), synth.mamba_block_weights(W, DEV, 2)]
    out, n_left, infos = blocks.run_blocks(kinds, wts, hidden, W.N, W.M, budgets, W.mamba, W.attn)
    assert n_left == budgets[-1] and not infos[0] and infos[1] and infos[2]
    h_dev, n = hidden, W.N
    for l, (kind, wt, K) in enumerate(zip(kinds, wts, budgets)):
        if kind == "mamba":
            nxt, n_out, info = blocks.mamba_block(h_dev, n, W.M, wt, W.mamba, int(K))
        else:
            nxt, n_out, info = blocks.attn_block(h_dev, n, W.M, wt, W.attn, int(K))
        idx = info["idx"].cpu().numpy() if info else None
        if kind == "mamba":
            want, _ = ref.mamba_block(f(h_dev), n, W.M, _np(wt), W.mamba.H, W.mamba.P, W.mamba.G, W.mamba.n, "bf16", idx)
        else:
            want, _ = ref.attn_block(f(h_dev), n, W.M, _np(wt), W.attn.Hq, W.attn.Hkv, W.attn.d, "bf16", idx)
        assert_close(f(nxt), want, TOLB, "block %d output" % l)
        if info:
            assert torch.equal(info["idx"], infos[l]["idx"])
        h_dev, n = nxt, n_out
    assert torch.equal(h_dev, out), "run_blocks must chain the blocks unchanged"
    # a reducing block's indices refer to the rows that reached it
    assert int(infos[2]["idx"].max()) < budgets[1]
