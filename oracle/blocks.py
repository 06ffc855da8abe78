"""Reference blocks for the hidden-to-hidden tests -- TEST INFRASTRUCTURE, like the rest of this
package.  The same sequence of definitions as the library's blocks, composed from the oracle's
fp64 routines and numpy matrix products, with every tensor the device stores in a narrower type
rounded to that type at the same point (so both sides feed identical operands forward and the
comparison isolates each stage's arithmetic).  The kept-index list of a reducing block is an
input: selection parity is checked where the scores are.
"""
from __future__ import annotations

import numpy as np
import torch

from . import (attn, compact, conv1d_silu, gated_rmsnorm, rmsnorm, softplus_dt, ssd_seq)


def _round(a, dtype):
    """a (fp64 numpy) rounded to the device's storage type and back to fp64."""
    if dtype == "f32":
        return np.asarray(a, np.float32).astype(np.float64)
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).double().numpy()


def mamba_block(hidden, N, M, wt, H, P, G, n, dtype, idx=None, eps=1e-5):
    """hidden, wt[...]: fp64 numpy of the device's (already rounded) values; idx: kept vision tokens or None."""
    r = lambda a: _round(a, dtype)
    T = N + M
    d_inner, gn = H * P, G * n
    u = r(rmsnorm(hidden, wt["norm_w"], eps))
    z = r(u @ wt["W_z"])
    xbcdt = r(u @ wt["W_xbcdt"])
    xbc = r(conv1d_silu(xbcdt[:, :d_inner + 2 * gn], wt["conv_w"], wt["conv_b"]))
    dt = np.asarray(softplus_dt(xbcdt[:, d_inner + 2 * gn:], wt["dt_bias"]), np.float32).astype(np.float64)
    x, B, C = xbc[:, :d_inner].reshape(T, H, P), xbc[:, d_inner:d_inner + gn].reshape(T, G, n), \
        xbc[:, d_inner + gn:].reshape(T, G, n)
    pre = {"B": B, "C": C, "dt": dt}
    if idx is not None:
        x, B, C, dt, z, hidden = (compact(a, idx, N, M)[0] for a in (x, B, C, dt, z, hidden))
        T = idx.shape[0] + M
    y, _ = ssd_seq(x, dt, wt["A"], B, C, wt["D"])
    y = r(y)
    g = r(gated_rmsnorm(y.reshape(T, d_inner), z, wt["gnorm_w"], G, eps))
    return r(g @ wt["W_out"] + hidden), pre


def attn_block(hidden, N, M, wt, Hq, Hkv, d, dtype, idx=None, eps=1e-5):
    r = lambda a: _round(a, dtype)
    T = N + M
    u = r(rmsnorm(hidden, wt["norm_w"], eps))
    q = r(u @ wt["W_q"]).reshape(T, Hq, d)
    k = r(u @ wt["W_k"]).reshape(T, Hkv, d)
    v = r(u @ wt["W_v"]).reshape(T, Hkv, d)
    pre = {"q": q, "k": k}
    if idx is not None:
        q, k, v, hidden = (compact(a, idx, N, M)[0] for a in (q, k, v, hidden))
        T = idx.shape[0] + M
    o = r(attn(q, k, v))
    return r(o.reshape(T, Hq * d) @ wt["W_o"] + hidden), pre
