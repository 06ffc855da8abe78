"""Progressive low-to-high reduction over a stack of hybrid layers (paper Sec. 3.2): layer l keeps
K_l = schedule_budgets(alpha)[l] vision tokens; the reducing layer scores with its own b/c/dt or
q/k, runs its mixer on the survivors, and every later layer only sees the survivors.

"Tape mode": each layer's mixer inputs are given at full length (synthetic stand-ins for the
projections of that layer's hidden states) and gathered through the composed position map, so the
stack exercises score -> select -> compact -> mixer, the composition of index maps and the
budgets, without the block glue (projections, norms, FFN) that is outside this library.
Orchestration only: every tensor operation is a call into the C library.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import torch

from . import binding as strd


def run_stack(kinds: Sequence[str], layer_inputs: Sequence[Dict[str, torch.Tensor]], hidden: torch.Tensor,
              N: int, M: int, budgets: Sequence[int], chunk: int = 256) -> List[Dict[str, torch.Tensor]]:
    """kinds[l] in {"mamba", "attn"}; layer_inputs[l] holds full-length x,B,C,dt,A or q,k,v;
    budgets[l] = vision tokens layer l runs on (non-increasing).  Returns per layer the mixer
    output, the scores / kept indices of a reducing layer and the position map in force."""
    dev = hidden.device
    pos = torch.arange(N + M, dtype=torch.int32, device=dev)   # original position of every current row
    n_cur = N
    out = []
    for l, kind in enumerate(kinds):
        t = layer_inputs[l]
        keys = ("x", "B", "C", "dt") if kind == "mamba" else ("q", "k", "v")
        if n_cur < N:   # this layer's tensors restricted to the rows that survived earlier layers
            cur, _ = strd.compact_batch([t[k] for k in keys], pos[:n_cur].contiguous(), N, M)
        else:
            cur = [t[k] for k in keys]
        cur = dict(zip(keys, cur))
        rec: Dict[str, torch.Tensor] = {}
        K = int(budgets[l])
        if K < n_cur:
            if kind == "mamba":
                s = strd.score_mamba(cur["B"][:n_cur].contiguous(), cur["C"][n_cur:].contiguous(),
                                     cur["dt"][:n_cur].contiguous())
            else:
                s = strd.score_attn(cur["q"][n_cur:].contiguous(), cur["k"][:n_cur].contiguous())
            idx = strd.select_topk(s, K)
            kept, pos = strd.compact_batch([cur[k] for k in keys] + [hidden], idx, n_cur, M, pos_in=pos)
            cur = dict(zip(keys, kept[:-1]))
            hidden = kept[-1]
            rec["scores"], rec["idx"] = s, idx
            n_cur = K
        if kind == "mamba":
            y, S = strd.ssd_prefill(cur["x"], cur["dt"], t["A"], cur["B"], cur["C"], chunk=chunk)
            rec["y"], rec["state"] = y, S
        else:
            rec["y"] = strd.attn_prefill(cur["q"], cur["k"], cur["v"])
        rec["pos"] = pos
        out.append(rec)
    return out


def model_stack_time(types: Sequence[int], budgets: Sequence[int], N0: int, mixer_time, reduce_time):
    """Time of the mixers of a hybrid stack under a schedule, from measured per-layer times.

    types[l]: binding.LAYER_*; budgets[l]: vision tokens layer l runs on (schedule_budgets);
    mixer_time(kind, n_vis) and reduce_time(kind, n_in, k): measured seconds of the layer mixer on
    n_vis vision (+ text) tokens and of score + select + compact from n_in to k vision tokens, kind in
    {"mamba", "attn"}.  A layer reduces when its budget is below what the previous layer left;
    MLP layers cannot score, so their budget change is carried to the next Mamba / attention layer
    (their own cost is not modelled: no MLP kernel is part of this library).
    Returns (reduced_seconds, full_seconds)."""
    n_cur, red, full = N0, 0.0, 0.0
    for ty, k in zip(types, budgets):
        if ty == strd.LAYER_MLP:
            continue
        kind = "attn" if ty == strd.LAYER_ATTN else "mamba"
        if k < n_cur:
            red += reduce_time(kind, n_cur, k)
            n_cur = k
        red += mixer_time(kind, n_cur)
        full += mixer_time(kind, N0)
    return red, full
