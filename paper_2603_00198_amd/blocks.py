"""Hidden-to-hidden blocks of a hybrid layer stack with token reduction inside: pre-norm, projections, the Mamba-2 glue (short causal convolution + SiLU on x, B, C;
softplus on dt; gated RMS norm) or the attention glue, the mixer on the surviving tokens, the
out-projection added to the residual stream.  A reducing block scores with its own projected
b, c, dt (or q, k) -- after the convolution -- keeps the top K vision tokens and compacts what the
rest of the block and the later blocks read, the residual stream included (paper Sec. 3.1, 3.2).
Projections whose outputs nothing reads before the selection (the gate z; the queries and values of
the vision tokens) are taken after it, of the kept rows only.

The paper builds on the Mamba-2 block and a standard pre-norm attention block without restating
them; the attention block here carries no positional encoding.  Orchestration only: every tensor
operation is a call into the C library.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence, Tuple

import torch

from . import binding as strd
from .synth import AttnShape, MambaShape


def mamba_block(hidden: torch.Tensor, N: int, M: int, wt: Dict[str, torch.Tensor], s: MambaShape,
                K: Optional[int] = None, eps: float = 1e-5) -> Tuple[torch.Tensor, int, Dict[str, torch.Tensor]]:
    """hidden [N+M, d_model] -> (hidden' [N'+M, d_model], N', info); N' = K if the block reduces."""
    T = N + M
    d_inner, gn = s.H * s.P, s.G * s.n
    u = strd.rmsnorm(hidden, wt["norm_w"], eps)
    xbcdt = strd.linear(u, wt["W_xbcdt"])
    x, B, C = strd.conv1d_silu(xbcdt, wt["conv_w"], wt["conv_b"], d_inner, gn)
    dt = strd.softplus_dt(xbcdt[:, d_inner + 2 * gn:], wt["dt_bias"])
    x, B, C = x.view(T, s.H, s.P), B.view(T, s.G, s.n), C.view(T, s.G, s.n)
    info: Dict[str, torch.Tensor] = {}
    if K is not None and K < N:
        scores = strd.score_mamba(B[:N], C[N:], dt[:N])
        idx = strd.select_topk(scores, K)
        # the gate z is read only after the scan: its projection is a row-wise product, so it is taken of the
        # kept rows of u alone (the same values as projecting every row and compacting, at K + M rows' cost)
        (x, B, C, dt, u, hidden), _ = strd.compact_batch([x, B, C, dt, u, hidden], idx, N, M)
        info = {"scores": scores, "idx": idx}
        N, T = K, K + M
    z = strd.linear(u, wt["W_z"])
    y, _ = strd.ssd_prefill(x, dt, wt["A"], B, C, wt["D"], chunk=s.chunk, want_state=False)
    gated = strd.gated_rmsnorm(y.view(T, d_inner), z, wt["gnorm_w"], s.G, eps)
    return strd.linear(gated, wt["W_out"], residual=hidden), N, info


def attn_block(hidden: torch.Tensor, N: int, M: int, wt: Dict[str, torch.Tensor], s: AttnShape,
               K: Optional[int] = None, eps: float = 1e-5) -> Tuple[torch.Tensor, int, Dict[str, torch.Tensor]]:
    T = N + M
    u = strd.rmsnorm(hidden, wt["norm_w"], eps)
    k = strd.linear(u, wt["W_k"]).view(T, s.Hkv, s.d)
    info: Dict[str, torch.Tensor] = {}
    if K is not None and K < N:
        # the score needs the keys of every vision token but the queries of the text rows only; the queries
        # and values of the vision tokens are projected after the selection, of the kept rows of u alone
        # (row-wise products: the same values as projecting every row and compacting)
        q_txt = strd.linear(u[N:], wt["W_q"]).view(M, s.Hq, s.d)
        scores = strd.score_attn(q_txt, k[:N])
        idx = strd.select_topk(scores, K)
        (k, u, hidden), _ = strd.compact_batch([k, u, hidden], idx, N, M)
        info = {"scores": scores, "idx": idx}
        N, T = K, K + M
    q = strd.linear(u, wt["W_q"]).view(T, s.Hq, s.d)
    v = strd.linear(u, wt["W_v"]).view(T, s.Hkv, s.d)
    o = strd.attn_prefill(q, k, v)
    return strd.linear(o.view(T, s.Hq * s.d), wt["W_o"], residual=hidden), N, info


def run_blocks(kinds: Sequence[str], weights: Sequence[Dict[str, torch.Tensor]], hidden: torch.Tensor, N: int, M: int,
               budgets: Sequence[int], mamba: Optional[MambaShape] = None, attn: Optional[AttnShape] = None):
    """kinds[l] in {"mamba", "attn"}; budgets[l] = vision tokens block l runs its mixer on
    (non-increasing).  Returns the final hidden states, the vision tokens left, and per-block info."""
    infos = []
    for kind, wt, K in zip(kinds, weights, budgets):
        if kind == "mamba":
            hidden, N, info = mamba_block(hidden, N, M, wt, mamba, int(K))
        else:
            hidden, N, info = attn_block(hidden, N, M, wt, attn, int(K))
        infos.append(info)
    return hidden, N, infos
