"""CPU fp64 oracle for the token-reduced prefill path -- TEST INFRASTRUCTURE.

Thin ctypes/numpy marshalling around ``strd_oracle.c`` (plain fp64 loops written
from the paper's equations).  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product package never does, and
this package never imports the product.

Every function takes numpy arrays (any float dtype; converted exactly to
float64) in the token-major layouts named in the C source and returns new
float64 / int32 arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "strd_oracle.c")
_LIB = os.path.join(_HERE, "libstrd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (CPU only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, name):
    if rc != 0:
        raise ValueError("%s: oracle returned %d" % (name, rc))


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle will use."""
    return int(os.environ.get("OMP_NUM_THREADS") or len(os.sched_getaffinity(0)))


def score_attn(q_txt, k_vis, scale=None):
    q, k = _f64(q_txt), _f64(k_vis)
    M, Hq, d = q.shape
    N, Hkv, d2 = k.shape
    assert d == d2
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    s = np.empty(N, np.float64)
    _check(_load().oracle_score_attn(_p(q), _p(k), _p(s), M, N, Hq, Hkv, d, ctypes.c_double(scale)),
           "score_attn")
    return s


def score_mamba(B_vis, C_txt, dt_vis):
    B, C, dt = _f64(B_vis), _f64(C_txt), _f64(dt_vis)
    N, G, n = B.shape
    M = C.shape[0]
    H = dt.shape[1]
    assert C.shape[1:] == (G, n) and dt.shape[0] == N
    s = np.empty(N, np.float64)
    _check(_load().oracle_score_mamba(_p(B), _p(C), _p(dt), _p(s), M, N, H, G, n), "score_mamba")
    return s


def score_mamba_full(B_all, C_all, dt_all, A, N, rows=None):
    """Full Mamba Dynamic score |w_{t,j}| averaged over text rows and heads (optionally only for
    the vision tokens listed in rows)."""
    B, C, dt, A = _f64(B_all), _f64(C_all), _f64(dt_all), _f64(A)
    T, G, n = B.shape
    M = T - N
    H = dt.shape[1]
    if rows is None:
        s = np.empty(N, np.float64)
        _check(_load().oracle_score_mamba_full(_p(B), _p(C), _p(dt), _p(A), _p(s), M, N, H, G, n),
               "score_mamba_full")
        return s
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    s = np.empty(rows.shape[0], np.float64)
    _check(_load().oracle_score_mamba_full_rows(_p(B), _p(C), _p(dt), _p(A), _p(s), M, N, H, G, n, _p(rows),
                                                int(rows.shape[0])), "score_mamba_full_rows")
    return s


def select_topk(scores, K):
    s = _f64(scores)
    idx = np.empty(K, np.int32)
    _check(_load().oracle_select_topk(_p(s), s.shape[0], int(K), _p(idx)), "select_topk")
    return idx


def compact(src, idx, N, M, pos_in=None):
    """Row gather of a [N+M, ...] array of any dtype; returns (dst, pos_out)."""
    src = np.ascontiguousarray(src)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    K = idx.shape[0]
    assert src.shape[0] == N + M
    row_bytes = src.strides[0] if src.ndim > 1 else src.itemsize
    if src.shape[0] == 0:
        row_bytes = int(np.prod(src.shape[1:])) * src.itemsize
    dst = np.empty((K + M,) + src.shape[1:], src.dtype)
    pos_out = np.empty(K + M, np.int32)
    pin = None if pos_in is None else np.ascontiguousarray(pos_in, dtype=np.int32)
    _check(_load().oracle_compact(_p(src), _p(idx), _p(dst), N, M, K, ctypes.c_int64(row_bytes),
                                  _p(pin), _p(pos_out)), "compact")
    return dst, pos_out


def _ssd_args(x, dt, A, B, C, D, S_in):
    x, dt, A, B, C = _f64(x), _f64(dt), _f64(A), _f64(B), _f64(C)
    T, H, P = x.shape
    G, n = B.shape[1:]
    assert dt.shape == (T, H) and A.shape == (H,) and C.shape == (T, G, n)
    D = None if D is None else _f64(D)
    S_in = None if S_in is None else _f64(S_in)
    if S_in is not None:
        assert S_in.shape == (H, P, n)
    return x, dt, A, B, C, D, S_in, T, H, P, G, n


def ssd_seq(x, dt, A, B, C, D=None, S_in=None):
    """Token-by-token recurrence; returns (y [T,H,P], S_out [H,P,n])."""
    x, dt, A, B, C, D, S_in, T, H, P, G, n = _ssd_args(x, dt, A, B, C, D, S_in)
    y = np.empty((T, H, P), np.float64)
    S_out = np.empty((H, P, n), np.float64)
    _check(_load().oracle_ssd_seq(_p(x), _p(dt), _p(A), _p(B), _p(C), _p(D), _p(S_in), _p(y),
                                  _p(S_out), T, H, P, G, n), "ssd_seq")
    return y, S_out


def ssd_unrolled(x, dt, A, B, C, D=None, S_in=None):
    x, dt, A, B, C, D, S_in, T, H, P, G, n = _ssd_args(x, dt, A, B, C, D, S_in)
    y = np.empty((T, H, P), np.float64)
    _check(_load().oracle_ssd_unrolled(_p(x), _p(dt), _p(A), _p(B), _p(C), _p(D), _p(S_in), _p(y),
                                       T, H, P, G, n), "ssd_unrolled")
    return y


def ssd_chunked(x, dt, A, B, C, D=None, S_in=None, chunk=64):
    x, dt, A, B, C, D, S_in, T, H, P, G, n = _ssd_args(x, dt, A, B, C, D, S_in)
    y = np.empty((T, H, P), np.float64)
    S_out = np.empty((H, P, n), np.float64)
    _check(_load().oracle_ssd_chunked(_p(x), _p(dt), _p(A), _p(B), _p(C), _p(D), _p(S_in), _p(y),
                                      _p(S_out), T, H, P, G, n, int(chunk)), "ssd_chunked")
    return y, S_out


def attn(q, k, v, scale=None, rows=None):
    """Causal GQA attention; ``rows`` (int array) limits the output to those query rows."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    assert k.shape == (T, Hkv, d) and v.shape == (T, Hkv, d)
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    if rows is None:
        r, nrows = None, T
    else:
        r = np.ascontiguousarray(rows, dtype=np.int32)
        nrows = r.shape[0]
    o = np.empty((nrows, Hq, d), np.float64)
    _check(_load().oracle_attn(_p(q), _p(k), _p(v), _p(o), T, Hq, Hkv, d, ctypes.c_double(scale),
                               _p(r), nrows), "attn")
    return o


# ------------------------------------------------------------------ block glue -------------
def rmsnorm(x, w, eps=1e-5):
    x, w = _f64(x), _f64(w)
    out = np.empty_like(x)
    _check(_load().oracle_rmsnorm(_p(x), _p(w), _p(out), x.shape[0], x.shape[1], ctypes.c_double(eps)), "rmsnorm")
    return out


def gated_rmsnorm(y, z, w, groups=1, eps=1e-5):
    y, z, w = _f64(y), _f64(z), _f64(w)
    out = np.empty_like(y)
    _check(_load().oracle_gated_rmsnorm(_p(y), _p(z), _p(w), _p(out), y.shape[0], y.shape[1], int(groups),
                                        ctypes.c_double(eps)), "gated_rmsnorm")
    return out


def conv1d_silu(xbc, w, b=None):
    """Causal depthwise conv + SiLU over all columns of xbc [T,C]; w [C,W], b [C] or None."""
    xbc, w = _f64(xbc), _f64(w)
    b = None if b is None else _f64(b)
    out = np.empty_like(xbc)
    _check(_load().oracle_conv1d_silu(_p(xbc), _p(w), _p(b), _p(out), xbc.shape[0], xbc.shape[1], w.shape[1]),
           "conv1d_silu")
    return out


def softplus_dt(raw, bias=None):
    raw = _f64(raw)
    bias = None if bias is None else _f64(bias)
    out = np.empty_like(raw)
    _check(_load().oracle_softplus_dt(_p(raw), _p(bias), _p(out), raw.shape[0], raw.shape[1]), "softplus_dt")
    return out


# ------------------------------------------------------------------ variants ---------------
def avgpool(src, N, M, K, pos_in=None):
    """Average-pool reduction of the N vision rows of src [N+M, D] to K rows; returns (dst, pos_out)."""
    src = _f64(src)
    assert src.ndim == 2 and src.shape[0] == N + M
    dst = np.empty((K + M, src.shape[1]), np.float64)
    pos_out = np.empty(K + M, np.int32)
    pin = None if pos_in is None else np.ascontiguousarray(pos_in, dtype=np.int32)
    _check(_load().oracle_avgpool(_p(src), _p(dst), N, M, K, src.shape[1], _p(pin), _p(pos_out)), "avgpool")
    return dst, pos_out


def ssd_decode_step(x1, dt1, A, B1, C1, D, S):
    """One token of the recurrence from the carried state S [H,P,n] (paper Eqs. ssm_state_update,
    ssm_output with T = 1); x1 [H,P], dt1 [H], B1, C1 [G,n].  Returns (y [H,P], S_new)."""
    y, S_new = ssd_seq(np.asarray(x1)[None], np.asarray(dt1)[None], A, np.asarray(B1)[None], np.asarray(C1)[None],
                       D=D, S_in=S)
    return y[0], S_new


def attn_decode_step(q1, k_cache, v_cache, scale=None):
    """The newest token's attention output over all T cached rows (its own included): the last row
    of causal attention.  q1 [Hq,d], k_cache, v_cache [T,Hkv,d]; returns [Hq,d]."""
    k, v = _f64(k_cache), _f64(v_cache)
    T = k.shape[0]
    q = np.zeros((T,) + np.asarray(q1).shape, np.float64)
    q[T - 1] = q1
    return attn(q, k, v, scale=scale, rows=[T - 1])[0]
