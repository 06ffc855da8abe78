"""ctypes binding of libstrd.so: same names as the C entry points, torch tensors in and out.

Only marshalling happens here: shape checks, output/workspace allocation through torch
(device memory plumbing) and the current HIP stream.  Every step of the path runs in the
library's kernels; if the library is missing the import of any function fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libstrd.so")

STRD_F32, STRD_BF16 = 0, 1
_c = ctypes
_vp, _int, _i64, _f32, _sz = _c.c_void_p, _c.c_int, _c.c_int64, _c.c_float, _c.c_size_t

_SIGNATURES = {
    "strd_status_string": (_c.c_char_p, [_int]),
    "strd_version": (_int, []),
    "strd_score_attn_kernel_path": (_int, [_int] * 6),
    "strd_score_mamba_kernel_path": (_int, [_int] * 6),
    "strd_ssd_prefill_kernel_path": (_int, [_int] * 6),
    "strd_attn_prefill_kernel_path": (_int, [_int] * 5),
    "strd_score_attn_workspace": (_sz, [_int] * 5 + [_int]),
    "strd_score_attn": (_int, [_vp, _vp, _vp] + [_int] * 5 + [_f32, _int, _vp, _sz, _vp]),
    "strd_score_mamba_workspace": (_sz, [_int] * 5 + [_int]),
    "strd_score_mamba": (_int, [_vp, _vp, _vp, _vp] + [_int] * 5 + [_int, _vp, _sz, _vp]),
    "strd_score_mamba_full_workspace": (_sz, [_int] * 5 + [_int]),
    "strd_score_mamba_full": (_int, [_vp] * 5 + [_int] * 5 + [_int, _vp, _sz, _vp]),
    "strd_select_topk_workspace": (_sz, [_int, _int]),
    "strd_select_topk": (_int, [_vp, _int, _int, _vp, _vp, _sz, _vp]),
    "strd_select_topk_noalloc_max_n": (_int, []),
    "strd_select_topk_noalloc": (_int, [_vp, _int, _int, _vp, _vp]),
    "strd_compact": (_int, [_vp, _vp, _vp, _int, _int, _int, _i64, _vp, _vp, _vp]),
    "strd_compact_batch": (_int, [_vp, _int, _vp, _int, _int, _int, _vp, _vp, _vp]),
    "strd_mfma_rate_probe": (_int, [_vp, _int, _int, _int, _vp]),
    "strd_score_attn_varlen_workspace": (_sz, [_vp, _int, _int, _int, _int, _int]),
    "strd_score_attn_varlen": (_int, [_vp, _vp, _vp, _int, _vp, _int, _int, _int, _int, _f32, _int, _vp, _sz, _vp]),
    "strd_score_mamba_varlen_workspace": (_sz, [_vp, _int, _int, _int, _int, _int]),
    "strd_score_mamba_varlen": (_int, [_vp, _vp, _vp, _vp, _int, _vp, _int, _int, _int, _int, _int, _vp, _sz, _vp]),
    "strd_select_topk_varlen_max_n": (_int, []),
    "strd_select_topk_varlen": (_int, [_vp, _int, _vp, _int, _vp, _vp]),
    "strd_compact_varlen": (_int, [_vp, _int, _vp, _vp, _int, _vp, _vp, _vp]),
    "strd_ssd_prefill_workspace": (_sz, [_int] * 6 + [_int]),
    "strd_ssd_prefill": (_int, [_vp] * 9 + [_int] * 6 + [_int, _vp, _sz, _vp]),
    "strd_ssd_prefill_gather": (_int, [_vp] * 10 + [_int] * 8 + [_int, _vp, _sz, _vp]),
    "strd_attn_prefill_workspace": (_sz, [_int] * 4 + [_int]),
    "strd_attn_prefill": (_int, [_vp] * 4 + [_int] * 4 + [_f32, _int, _vp, _sz, _vp]),
    "strd_linear": (_int, [_vp, _vp, _vp, _vp, _int, _int, _int, _int, _vp]),
    "strd_linear_mfma": (_int, [_vp, _vp, _vp, _vp, _int, _int, _int, _int, _vp]),
    "strd_linear_library": (_int, [_vp, _vp, _vp, _vp, _int, _int, _int, _int, _vp]),
    "strd_linear_mfma_supported": (_int, [_int, _int, _int, _int]),
    "strd_rmsnorm": (_int, [_vp, _vp, _vp, _int, _int, _f32, _int, _vp]),
    "strd_gated_rmsnorm": (_int, [_vp, _vp, _int, _vp, _vp, _int, _int, _int, _f32, _int, _vp]),
    "strd_conv1d_silu": (_int, [_vp, _int, _vp, _vp, _vp, _vp, _vp] + [_int] * 4 + [_int, _vp]),
    "strd_softplus_dt": (_int, [_vp, _int, _int, _vp, _vp, _int, _int, _int, _vp]),
    "strd_avgpool": (_int, [_vp, _vp, _int, _int, _int, _int, _int, _vp, _vp, _vp]),
    "strd_ssd_decode_step": (_int, [_vp] * 8 + [_int] * 4 + [_int, _vp]),
    "strd_attn_decode_step_workspace": (_c.c_size_t, [_int, _int, _int, _int, _int]),
    "strd_attn_decode_step": (_int, [_vp, _vp, _vp, _vp, _int, _int, _int, _int, _f32, _int, _vp, _c.c_size_t, _vp]),
    "strd_schedule_budgets": (_int, [_vp, _int, _int, _int, _vp]),
    "strd_schedule_sigmoid": (_int, [_int, _c.c_double, _c.c_double, _c.c_double, _c.c_double, _vp]),
    "strd_schedule_step_decay": (_int, [_vp, _vp, _vp, _int, _int, _vp]),
    "strd_hybrid_layout": (_int, [_int, _vp]),
    "strd_schedule_named": (_int, [_c.c_char_p, _vp]),
}

_lib = None


class StrdError(RuntimeError):
    pass


def lib():
    """The loaded C library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise StrdError("%s is missing: run `python -m paper_2603_00198_amd.build` "
                            "(there is no fallback path)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def exported_symbols() -> Sequence[str]:
    return tuple(_SIGNATURES)


PATH_NONE, PATH_MFMA, PATH_SIMT = 0, 1, 2


def kernel_path(op: str, *sizes: int, dtype: torch.dtype = torch.bfloat16) -> int:
    """PATH_MFMA / PATH_SIMT / PATH_NONE for op in {"score_attn", "score_mamba", "ssd_prefill",
    "attn_prefill"} with the size arguments of that entry point (host only)."""
    io = STRD_BF16 if dtype == torch.bfloat16 else STRD_F32
    return getattr(lib(), "strd_%s_kernel_path" % op)(*[int(v) for v in sizes], io)


def _check(rc: int, what: str):
    if rc != 0:
        raise StrdError("%s failed: %s" % (what, lib().strd_status_string(rc).decode()))


def _io(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return STRD_F32
    if t.dtype == torch.bfloat16:
        return STRD_BF16
    raise StrdError("unsupported tensor dtype %s (fp32 or bf16)" % t.dtype)


def _dev(*ts: Optional[torch.Tensor]):
    for t in ts:
        if t is None:
            continue
        if not t.is_cuda:
            raise StrdError("tensors must live on the GPU")
        if not t.is_contiguous():
            raise StrdError("tensors must be contiguous")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ws(nbytes: int, like: torch.Tensor) -> Tuple[Optional[torch.Tensor], int]:
    if nbytes == 0:
        return None, 0
    return torch.empty(nbytes, dtype=torch.uint8, device=like.device), nbytes


def score_attn(q_txt: torch.Tensor, k_vis: torch.Tensor, scale: Optional[float] = None,
               out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """s[N] fp32 from text queries [M,Hq,d] and vision keys [N,Hkv,d]."""
    _dev(q_txt, k_vis, out, ws)
    M, Hq, d = q_txt.shape
    N, Hkv, d2 = k_vis.shape
    if d != d2 or q_txt.dtype != k_vis.dtype:
        raise StrdError("q/k mismatch")
    io = _io(q_txt)
    if scale is None:
        scale = d ** -0.5
    if out is None:
        out = torch.empty(N, dtype=torch.float32, device=q_txt.device)
    need = lib().strd_score_attn_workspace(M, N, Hq, Hkv, d, io)
    if ws is None:
        ws, _ = _ws(need, q_txt)
    _check(lib().strd_score_attn(_ptr(q_txt), _ptr(k_vis), _ptr(out), M, N, Hq, Hkv, d, scale, io,
                                 _ptr(ws), 0 if ws is None else ws.numel(), _stream()), "score_attn")
    return out


def score_mamba(B_vis: torch.Tensor, C_txt: torch.Tensor, dt_vis: torch.Tensor,
                out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """s[N] fp32 from vision b [N,G,n], text c [M,G,n] and vision dt [N,H] (fp32)."""
    _dev(B_vis, C_txt, dt_vis, out, ws)
    N, G, n = B_vis.shape
    M = C_txt.shape[0]
    H = dt_vis.shape[1]
    if C_txt.shape[1:] != (G, n) or dt_vis.shape[0] != N or dt_vis.dtype != torch.float32 \
            or B_vis.dtype != C_txt.dtype:
        raise StrdError("B/C/dt mismatch")
    io = _io(B_vis)
    if out is None:
        out = torch.empty(N, dtype=torch.float32, device=B_vis.device)
    need = lib().strd_score_mamba_workspace(M, N, H, G, n, io)
    if ws is None:
        ws, _ = _ws(need, B_vis)
    _check(lib().strd_score_mamba(_ptr(B_vis), _ptr(C_txt), _ptr(dt_vis), _ptr(out), M, N, H, G, n, io,
                                  _ptr(ws), 0 if ws is None else ws.numel(), _stream()), "score_mamba")
    return out


def score_mamba_full(B_vis: torch.Tensor, C_txt: torch.Tensor, dt_all: torch.Tensor, A: torch.Tensor,
                     out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Full Mamba Dynamic score s[N] fp32 from vision b [N,G,n], text c [M,G,n], dt of all tokens
    [N+M,H] (fp32, vision rows first) and A [H]."""
    _dev(B_vis, C_txt, dt_all, A, out, ws)
    N, G, n = B_vis.shape
    M = C_txt.shape[0]
    H = dt_all.shape[1]
    if C_txt.shape[1:] != (G, n) or dt_all.shape[0] != N + M or dt_all.dtype != torch.float32 \
            or A.shape != (H,) or A.dtype != torch.float32 or B_vis.dtype != C_txt.dtype:
        raise StrdError("B/C/dt/A mismatch")
    io = _io(B_vis)
    if out is None:
        out = torch.empty(N, dtype=torch.float32, device=B_vis.device)
    need = lib().strd_score_mamba_full_workspace(M, N, H, G, n, io)
    if ws is None:
        ws, _ = _ws(need, B_vis)
    _check(lib().strd_score_mamba_full(_ptr(B_vis), _ptr(C_txt), _ptr(dt_all), _ptr(A), _ptr(out), M, N, H, G, n, io,
                                       _ptr(ws), 0 if ws is None else ws.numel(), _stream()), "score_mamba_full")
    return out


def select_topk(scores: torch.Tensor, K: int, out: Optional[torch.Tensor] = None,
                ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """idx[K] int32 ascending: the K highest scores, ties to the lowest index."""
    _dev(scores, out, ws)
    if scores.dtype != torch.float32 or scores.dim() != 1:
        raise StrdError("scores must be a 1-D fp32 tensor")
    N = scores.shape[0]
    if out is None:
        out = torch.empty(K, dtype=torch.int32, device=scores.device)
    need = lib().strd_select_topk_workspace(N, K)
    if ws is None:
        ws, _ = _ws(need, scores)
    _check(lib().strd_select_topk(_ptr(scores), N, K, _ptr(out), _ptr(ws), 0 if ws is None else ws.numel(),
                                  _stream()), "select_topk")
    return out


def select_topk_noalloc(scores: torch.Tensor, K: int, out: torch.Tensor) -> torch.Tensor:
    """select_topk through the entry point that allocates nothing: `out` [K] int32 is the caller's."""
    _dev(scores, out)
    if scores.dtype != torch.float32 or scores.dim() != 1 or out.dtype != torch.int32 or out.shape != (K,):
        raise StrdError("scores must be a 1-D fp32 tensor, out a [K] int32 tensor")
    _check(lib().strd_select_topk_noalloc(_ptr(scores), scores.shape[0], K, _ptr(out), _stream()), "select_topk_noalloc")
    return out


def compact(src: Optional[torch.Tensor], idx: torch.Tensor, N: int, M: int,
            pos_in: Optional[torch.Tensor] = None, want_pos: bool = False,
            out: Optional[torch.Tensor] = None):
    """Gather rows idx (vision) + the M text rows of src [N+M, ...]; returns dst or (dst, pos_out)."""
    _dev(src, idx, pos_in, out)
    if idx.dtype != torch.int32:
        raise StrdError("idx must be int32")
    K = idx.shape[0]
    dst, row_bytes = None, 0
    if src is not None:
        if src.shape[0] != N + M:
            raise StrdError("src must have N+M rows")
        row_bytes = (src.numel() // max(src.shape[0], 1)) * src.element_size() if src.shape[0] else 0
        if src.shape[0] == 0:
            row_bytes = int(torch.Size(src.shape[1:]).numel()) * src.element_size()
        dst = out if out is not None else torch.empty((K + M,) + tuple(src.shape[1:]), dtype=src.dtype,
                                                      device=src.device)
    pos_out = None
    if want_pos or pos_in is not None:
        pos_out = torch.empty(K + M, dtype=torch.int32, device=idx.device)
    _check(lib().strd_compact(_ptr(src), _ptr(idx), _ptr(dst), N, M, K, row_bytes, _ptr(pos_in), _ptr(pos_out),
                              _stream()), "compact")
    if pos_out is not None:
        return dst, pos_out
    return dst


class _CompactItem(ctypes.Structure):
    _fields_ = [("src", _vp), ("dst", _vp), ("row_bytes", _i64)]


def compact_batch(srcs: Sequence[torch.Tensor], idx: torch.Tensor, N: int, M: int,
                  pos_in: Optional[torch.Tensor] = None, want_pos: bool = False,
                  outs: Optional[Sequence[torch.Tensor]] = None):
    """One-launch gather of several [N+M, ...] tensors by the same idx; returns (dsts, pos_out or None)."""
    _dev(idx, pos_in, *srcs)
    if idx.dtype != torch.int32:
        raise StrdError("idx must be int32")
    K = idx.shape[0]
    if outs is None:
        outs = [torch.empty((K + M,) + tuple(t.shape[1:]), dtype=t.dtype, device=t.device) for t in srcs]
    _dev(*outs)
    items = (_CompactItem * max(len(srcs), 1))()
    for i, (t, o) in enumerate(zip(srcs, outs)):
        if t.shape[0] != N + M or o.shape[0] != K + M or o.dtype != t.dtype or o.shape[1:] != t.shape[1:]:
            raise StrdError("compact_batch: tensor %d has the wrong shape" % i)
        items[i].src, items[i].dst = t.data_ptr(), o.data_ptr()
        items[i].row_bytes = int(torch.Size(t.shape[1:]).numel()) * t.element_size()
    pos_out = torch.empty(K + M, dtype=torch.int32, device=idx.device) if (want_pos or pos_in is not None) else None
    _check(lib().strd_compact_batch(ctypes.cast(items, _vp), len(srcs), _ptr(idx), N, M, K, _ptr(pos_in),
                                    _ptr(pos_out), _stream()), "compact_batch")
    return list(outs), pos_out


def mfma_rate_probe(workgroups: int, iters: int, random_operands: bool, out: Optional[torch.Tensor] = None,
                    device="cuda", small_products: bool = False) -> torch.Tensor:
    """Launches the matrix-core rate probe (a measurement aid): workgroups * 4 * iters * 32 * 32768 flop, as
    32 x 32 x 16 products or (small_products) twice as many 16 x 16 x 32 ones."""
    if out is None:
        out = torch.empty(workgroups * 256, dtype=torch.float32, device=device)
    _dev(out)
    mode = int(bool(random_operands)) | (2 if small_products else 0)
    _check(lib().strd_mfma_rate_probe(_ptr(out), workgroups, iters, mode, _stream()), "mfma_rate_probe")
    return out


# ---- packed batches of sequences: `seqs` is a list of (N, M, K) per sequence ----------------
class _Seq(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int32), ("M", ctypes.c_int32), ("K", ctypes.c_int32)]


def _seq_array(seqs):
    arr = (_Seq * len(seqs))()
    for i, (n, m, k) in enumerate(seqs):
        arr[i].N, arr[i].M, arr[i].K = int(n), int(m), int(k)
    return arr


def _varlen_ld(seqs, ld):
    return (max(int(n) for n, _, _ in seqs) + 3) // 4 * 4 if ld is None else int(ld)


def score_attn_varlen(q_all: torch.Tensor, k_all: torch.Tensor, seqs, scale: Optional[float] = None,
                      ld: Optional[int] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores [nseq, ld] fp32 of a packed batch: q_all [rows,Hq,d], k_all [rows,Hkv,d]."""
    _dev(q_all, k_all, out)
    rows, Hq, d = q_all.shape
    Hkv = k_all.shape[1]
    if k_all.shape[0] != rows or k_all.shape[2] != d or q_all.dtype != k_all.dtype \
            or rows != sum(int(n) + int(m) for n, m, _ in seqs):
        raise StrdError("score_attn_varlen: q/k/seqs mismatch")
    io, ld, arr = _io(q_all), _varlen_ld(seqs, ld), _seq_array(seqs)
    if scale is None:
        scale = d ** -0.5
    if out is None:
        out = torch.zeros(len(seqs), ld, dtype=torch.float32, device=q_all.device)
    ws, nb = _ws(lib().strd_score_attn_varlen_workspace(ctypes.cast(arr, _vp), len(seqs), Hq, Hkv, d, io), q_all)
    _check(lib().strd_score_attn_varlen(_ptr(q_all), _ptr(k_all), _ptr(out), ld, ctypes.cast(arr, _vp), len(seqs), Hq, Hkv,
                                        d, scale, io, _ptr(ws), nb, _stream()), "score_attn_varlen")
    return out


def score_mamba_varlen(B_all: torch.Tensor, C_all: torch.Tensor, dt_all: torch.Tensor, seqs,
                       ld: Optional[int] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores [nseq, ld] fp32 of a packed batch: B_all, C_all [rows,G,n], dt_all [rows,H] fp32."""
    _dev(B_all, C_all, dt_all, out)
    rows, G, n = B_all.shape
    H = dt_all.shape[1]
    if C_all.shape != B_all.shape or dt_all.shape[0] != rows or dt_all.dtype != torch.float32 \
            or B_all.dtype != C_all.dtype or rows != sum(int(a) + int(m) for a, m, _ in seqs):
        raise StrdError("score_mamba_varlen: B/C/dt/seqs mismatch")
    io, ld, arr = _io(B_all), _varlen_ld(seqs, ld), _seq_array(seqs)
    if out is None:
        out = torch.zeros(len(seqs), ld, dtype=torch.float32, device=B_all.device)
    ws, nb = _ws(lib().strd_score_mamba_varlen_workspace(ctypes.cast(arr, _vp), len(seqs), H, G, n, io), B_all)
    _check(lib().strd_score_mamba_varlen(_ptr(B_all), _ptr(C_all), _ptr(dt_all), _ptr(out), ld, ctypes.cast(arr, _vp),
                                         len(seqs), H, G, n, io, _ptr(ws), nb, _stream()), "score_mamba_varlen")
    return out


def select_topk_varlen(scores: torch.Tensor, seqs, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """idx [sum K] int32: per sequence, the K_b best of scores[b, :N_b], ascending, local to the sequence."""
    _dev(scores, out)
    if scores.dtype != torch.float32 or scores.dim() != 2 or scores.shape[0] != len(seqs):
        raise StrdError("select_topk_varlen: scores must be fp32 [nseq, ld]")
    arr = _seq_array(seqs)
    if out is None:
        out = torch.empty(sum(int(k) for _, _, k in seqs), dtype=torch.int32, device=scores.device)
    _check(lib().strd_select_topk_varlen(_ptr(scores), scores.shape[1], ctypes.cast(arr, _vp), len(seqs), _ptr(out),
                                         _stream()), "select_topk_varlen")
    return out


def compact_varlen(srcs: Sequence[torch.Tensor], idx: torch.Tensor, seqs, pos_in: Optional[torch.Tensor] = None,
                   want_pos: bool = False):
    """One-launch gather of several packed [rows, ...] tensors; returns (dsts [sum(K+M), ...], pos_out or None)."""
    _dev(idx, pos_in, *srcs)
    rows = sum(int(n) + int(m) for n, m, _ in seqs)
    rows_out = sum(int(k) + int(m) for _, m, k in seqs)
    if idx.dtype != torch.int32 or idx.shape[0] != sum(int(k) for _, _, k in seqs):
        raise StrdError("compact_varlen: idx must be int32 [sum K]")
    outs = [torch.empty((rows_out,) + tuple(t.shape[1:]), dtype=t.dtype, device=t.device) for t in srcs]
    items = (_CompactItem * max(len(srcs), 1))()
    for i, (t, o) in enumerate(zip(srcs, outs)):
        if t.shape[0] != rows:
            raise StrdError("compact_varlen: tensor %d has the wrong number of rows" % i)
        items[i].src, items[i].dst = t.data_ptr(), o.data_ptr()
        items[i].row_bytes = int(torch.Size(t.shape[1:]).numel()) * t.element_size()
    pos_out = torch.empty(rows_out, dtype=torch.int32, device=idx.device) if (want_pos or pos_in is not None) else None
    arr = _seq_array(seqs)
    _check(lib().strd_compact_varlen(ctypes.cast(items, _vp), len(srcs), _ptr(idx), ctypes.cast(arr, _vp), len(seqs),
                                     _ptr(pos_in), _ptr(pos_out), _stream()), "compact_varlen")
    return outs, pos_out


def ssd_prefill(x: torch.Tensor, dt: torch.Tensor, A: torch.Tensor, B: torch.Tensor, C: torch.Tensor,
                D: Optional[torch.Tensor] = None, S_in: Optional[torch.Tensor] = None, chunk: int = 256,
                want_state: bool = True, out: Optional[torch.Tensor] = None,
                ws: Optional[torch.Tensor] = None):
    """Mamba-2 scan: returns (y [T,H,P], S_out [H,P,n] fp32 or None)."""
    _dev(x, dt, A, B, C, D, S_in, out, ws)
    T, H, P = x.shape
    G, n = B.shape[1:]
    if dt.shape != (T, H) or A.shape != (H,) or B.shape != (T, G, n) or C.shape != (T, G, n) \
            or dt.dtype != torch.float32 or A.dtype != torch.float32 or B.dtype != x.dtype or C.dtype != x.dtype:
        raise StrdError("ssd_prefill: inconsistent shapes or dtypes")
    for t, shp in ((D, (H,)), (S_in, (H, P, n))):
        if t is not None and (tuple(t.shape) != shp or t.dtype != torch.float32):
            raise StrdError("ssd_prefill: D / S_in must be fp32 of shape %s" % (shp,))
    io = _io(x)
    y = out if out is not None else torch.empty_like(x)
    S_out = torch.empty(H, P, n, dtype=torch.float32, device=x.device) if want_state else None
    need = lib().strd_ssd_prefill_workspace(T, H, P, G, n, chunk, io)
    if ws is None:
        ws, _ = _ws(need, x)
    _check(lib().strd_ssd_prefill(_ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(S_in), _ptr(y),
                                  _ptr(S_out), T, H, P, G, n, chunk, io, _ptr(ws),
                                  0 if ws is None else ws.numel(), _stream()), "ssd_prefill")
    return y, S_out


def ssd_prefill_gather(x: torch.Tensor, dt: torch.Tensor, A: torch.Tensor, B: torch.Tensor, C: torch.Tensor,
                       idx: torch.Tensor, N: int, M: int, D: Optional[torch.Tensor] = None,
                       S_in: Optional[torch.Tensor] = None, chunk: int = 256, want_state: bool = True,
                       out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """Mamba-2 scan over rows idx (vision) + the M text rows of the uncompacted inputs [N+M, ...]."""
    _dev(x, dt, A, B, C, D, S_in, idx, out, ws)
    Ttot, H, P = x.shape
    G, n = B.shape[1:]
    K = idx.shape[0]
    if Ttot != N + M or dt.shape != (Ttot, H) or A.shape != (H,) or B.shape != (Ttot, G, n) or C.shape != (Ttot, G, n) \
            or dt.dtype != torch.float32 or A.dtype != torch.float32 or B.dtype != x.dtype or C.dtype != x.dtype \
            or idx.dtype != torch.int32:
        raise StrdError("ssd_prefill_gather: inconsistent shapes or dtypes")
    io = _io(x)
    y = out if out is not None else torch.empty((K + M, H, P), dtype=x.dtype, device=x.device)
    S_out = torch.empty(H, P, n, dtype=torch.float32, device=x.device) if want_state else None
    if ws is None:
        ws, _ = _ws(lib().strd_ssd_prefill_workspace(K + M, H, P, G, n, chunk, io), x)
    _check(lib().strd_ssd_prefill_gather(_ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(S_in), _ptr(idx),
                                         _ptr(y), _ptr(S_out), N, M, K, H, P, G, n, chunk, io, _ptr(ws),
                                         0 if ws is None else ws.numel(), _stream()),
           "ssd_prefill_gather")
    return y, S_out


def attn_prefill(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, scale: Optional[float] = None,
                 out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Causal GQA attention: o [T,Hq,d]."""
    _dev(q, k, v, out, ws)
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    if k.shape != (T, Hkv, d) or v.shape != (T, Hkv, d) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise StrdError("attn_prefill: inconsistent shapes or dtypes")
    io = _io(q)
    if scale is None:
        scale = d ** -0.5
    o = out if out is not None else torch.empty_like(q)
    need = lib().strd_attn_prefill_workspace(T, Hq, Hkv, d, io)
    if ws is None:
        ws, _ = _ws(need, q)
    _check(lib().strd_attn_prefill(_ptr(q), _ptr(k), _ptr(v), _ptr(o), T, Hq, Hkv, d, scale, io, _ptr(ws),
                                   0 if ws is None else ws.numel(), _stream()), "attn_prefill")
    return o


def avgpool(src: torch.Tensor, N: int, M: int, K: int, pos_in: Optional[torch.Tensor] = None,
            want_pos: bool = False):
    """Average-pool the N vision rows of src [N+M, D] into K consecutive windows, keep the M text
    rows; returns dst [K+M, D] or (dst, pos_out)."""
    _dev(src, pos_in)
    if src.dim() != 2 or src.shape[0] != N + M:
        raise StrdError("avgpool: src must be [N+M, D]")
    dst = torch.empty((K + M, src.shape[1]), dtype=src.dtype, device=src.device)
    pos = torch.empty(K + M, dtype=torch.int32, device=src.device) if (want_pos or pos_in is not None) else None
    _check(lib().strd_avgpool(_ptr(src), _ptr(dst), N, M, K, src.shape[1], _io(src), _ptr(pos_in), _ptr(pos),
                              _stream()), "avgpool")
    return (dst, pos) if pos is not None else dst


def ssd_decode_step(x: torch.Tensor, dt: torch.Tensor, A: torch.Tensor, B: torch.Tensor, C: torch.Tensor,
                    D: Optional[torch.Tensor], S: torch.Tensor) -> torch.Tensor:
    """One token of the recurrence: x [H,P], dt [H] fp32, B, C [G,n], S [H,P,n] fp32 updated in
    place; returns y [H,P]."""
    _dev(x, dt, A, B, C, D, S)
    H, P = x.shape
    G, n = B.shape
    if dt.shape != (H,) or A.shape != (H,) or C.shape != (G, n) or S.shape != (H, P, n) or S.dtype != torch.float32 \
            or dt.dtype != torch.float32 or A.dtype != torch.float32 or B.dtype != x.dtype or C.dtype != x.dtype \
            or (D is not None and (D.shape != (H,) or D.dtype != torch.float32)):
        raise StrdError("ssd_decode_step: inconsistent shapes or dtypes")
    y = torch.empty_like(x)
    _check(lib().strd_ssd_decode_step(_ptr(x), _ptr(dt), _ptr(A), _ptr(B), _ptr(C), _ptr(D), _ptr(S), _ptr(y), H, P,
                                      G, n, _io(x), _stream()), "ssd_decode_step")
    return y


def attn_decode_step(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, scale: Optional[float] = None,
                     ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The newest token's attention over the T cached rows (its own included): q [Hq,d],
    k_cache, v_cache [T,Hkv,d]; returns o [Hq,d]."""
    _dev(q, k_cache, v_cache, ws)
    Hq, d = q.shape
    T, Hkv = k_cache.shape[:2]
    if k_cache.shape != (T, Hkv, d) or v_cache.shape != (T, Hkv, d) or k_cache.dtype != q.dtype \
            or v_cache.dtype != q.dtype:
        raise StrdError("attn_decode_step: inconsistent shapes or dtypes")
    io = _io(q)
    if scale is None:
        scale = d ** -0.5
    o = torch.empty_like(q)
    if ws is None:
        ws, _ = _ws(lib().strd_attn_decode_step_workspace(T, Hq, Hkv, d, io), q)
    _check(lib().strd_attn_decode_step(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(o), T, Hq, Hkv, d, scale, io,
                                       _ptr(ws), 0 if ws is None else ws.numel(), _stream()), "attn_decode_step")
    return o


def schedule_budgets(alpha: Sequence[float], N0: int, K_min: int = 0):
    """Per-layer budgets K_l from retention ratios alpha_l (host only)."""
    L = len(alpha)
    a = (ctypes.c_double * L)(*[float(v) for v in alpha])
    k = (ctypes.c_int32 * L)()
    _check(lib().strd_schedule_budgets(ctypes.cast(a, _vp), L, int(N0), int(K_min), ctypes.cast(k, _vp)),
           "schedule_budgets")
    return list(k)


def schedule_sigmoid(L: int, a_start: float = 1.0, a_end: float = 0.125, k: float = 20.0, x0: float = 0.11):
    """Sigmoid retention ratios alpha_l, l = 0..L-1 (host only)."""
    out = (ctypes.c_double * L)()
    _check(lib().strd_schedule_sigmoid(int(L), a_start, a_end, k, x0, ctypes.cast(out, _vp)), "schedule_sigmoid")
    return list(out)


# ------------------------------------------------------------------ block glue -------------
def _rows(t: torch.Tensor, what: str) -> int:
    """Row pitch in elements of a 2-D GPU tensor whose rows are contiguous (a column slice is fine)."""
    if not t.is_cuda:
        raise StrdError("tensors must live on the GPU")
    if t.dim() != 2 or t.stride(1) != 1:
        raise StrdError("%s: rows must be contiguous" % what)
    return t.stride(0)


def linear(x: torch.Tensor, w: torch.Tensor, residual: Optional[torch.Tensor] = None,
           out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x [T,Kd] . w [Kd,Nd] (+ residual [T,Nd]): the library's own kernel for large bf16 products, rocBLAS otherwise."""
    _dev(x, w, residual, out)
    T, Kd = x.shape
    Nd = w.shape[1]
    if w.shape[0] != Kd or w.dtype != x.dtype or (residual is not None and (residual.shape != (T, Nd) or
                                                                             residual.dtype != x.dtype)):
        raise StrdError("linear: x [T,Kd], w [Kd,Nd], residual [T,Nd], one dtype")
    out = out if out is not None else torch.empty((T, Nd), dtype=x.dtype, device=x.device)
    _check(lib().strd_linear(_ptr(x), _ptr(w), _ptr(residual), _ptr(out), T, Kd, Nd, _io(x), _stream()), "linear")
    return out


def _linear_by(entry: str, x, w, residual, out):
    _dev(x, w, residual, out)
    T, Kd = x.shape
    Nd = w.shape[1]
    if w.shape[0] != Kd or w.dtype != x.dtype or (residual is not None and (residual.shape != (T, Nd) or
                                                                             residual.dtype != x.dtype)):
        raise StrdError("%s: x [T,Kd], w [Kd,Nd], residual [T,Nd], one dtype" % entry)
    out = out if out is not None else torch.empty((T, Nd), dtype=x.dtype, device=x.device)
    _check(getattr(lib(), "strd_" + entry)(_ptr(x), _ptr(w), _ptr(residual), _ptr(out), T, Kd, Nd, _io(x), _stream()), entry)
    return out


def linear_mfma(x: torch.Tensor, w: torch.Tensor, residual: Optional[torch.Tensor] = None,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The same product by the library's own matrix-core kernel only (bf16; no handle, no allocation)."""
    return _linear_by("linear_mfma", x, w, residual, out)


def linear_library(x: torch.Tensor, w: torch.Tensor, residual: Optional[torch.Tensor] = None,
                   out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The same product by rocBLAS whatever the shape (to time the two side by side)."""
    return _linear_by("linear_library", x, w, residual, out)


def linear_mfma_supported(T: int, Kd: int, Nd: int, dtype: torch.dtype) -> bool:
    return bool(lib().strd_linear_mfma_supported(T, Kd, Nd, 1 if dtype == torch.bfloat16 else 0))


def rmsnorm(x: torch.Tensor, w: torch.Tensor, eps: float = 1e-5, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(x, w, out)
    T, d = x.shape
    if not x.is_contiguous() or w.shape != (d,) or w.dtype != x.dtype:
        raise StrdError("rmsnorm: x [T,d] contiguous, w [d] of the same dtype")
    out = out if out is not None else torch.empty_like(x)
    _check(lib().strd_rmsnorm(_ptr(x), _ptr(w), _ptr(out), T, d, eps, _io(x), _stream()), "rmsnorm")
    return out


def gated_rmsnorm(y: torch.Tensor, z: torch.Tensor, w: torch.Tensor, groups: int = 1, eps: float = 1e-5,
                  out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """rmsnorm(y * silu(z)) * w per group of channels; z may be a column slice of a wider matrix."""
    _dev(y, w, out)
    T, D = y.shape
    if not y.is_contiguous() or z.shape != (T, D) or w.shape != (D,) or z.dtype != y.dtype or w.dtype != y.dtype:
        raise StrdError("gated_rmsnorm: y, z [T,D], w [D], one dtype")
    out = out if out is not None else torch.empty_like(y)
    _check(lib().strd_gated_rmsnorm(_ptr(y), _ptr(z), _rows(z, "z"), _ptr(w), _ptr(out), T, D, groups, eps, _io(y),
                                    _stream()), "gated_rmsnorm")
    return out


def conv1d_silu(xbc: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], Cx: int, Cb: int):
    """Causal depthwise conv (w [Cx+2Cb, W]) + SiLU over the first Cx+2Cb columns of xbc (may be a
    column slice); returns contiguous x [T,Cx], B [T,Cb], C [T,Cb]."""
    _dev(w, b)
    T = xbc.shape[0]
    Ct = Cx + 2 * Cb
    if xbc.shape[1] < Ct or w.dim() != 2 or w.shape[0] != Ct or w.dtype != xbc.dtype or not w.is_contiguous() \
            or (b is not None and (b.shape != (Ct,) or b.dtype != xbc.dtype)):
        raise StrdError("conv1d_silu: xbc [T, >=Cx+2Cb], w [Cx+2Cb, W], b [Cx+2Cb], one dtype")
    e = lambda c: torch.empty((T, c), dtype=xbc.dtype, device=xbc.device)
    xo, Bo, Co = e(Cx), e(Cb), e(Cb)
    _check(lib().strd_conv1d_silu(_ptr(xbc), _rows(xbc, "xbc"), _ptr(w), _ptr(b), _ptr(xo), _ptr(Bo), _ptr(Co), T, Cx, Cb,
                                  w.shape[1], _io(xbc), _stream()), "conv1d_silu")
    return xo, Bo, Co


def softplus_dt(raw: torch.Tensor, bias: Optional[torch.Tensor] = None) -> torch.Tensor:
    """dt [T,H] fp32 = softplus(raw + bias); raw [T,H] may be a column slice, bias [H] fp32."""
    _dev(bias)
    T, H = raw.shape
    if bias is not None and (bias.shape != (H,) or bias.dtype != torch.float32):
        raise StrdError("softplus_dt: bias [H] fp32")
    dt = torch.empty((T, H), dtype=torch.float32, device=raw.device)
    _check(lib().strd_softplus_dt(_ptr(raw), _rows(raw, "raw"), 0, _ptr(bias), _ptr(dt), T, H, _io(raw), _stream()),
           "softplus_dt")
    return dt


HYBRID_LAYERS = 62
LAYER_MAMBA, LAYER_MLP, LAYER_ATTN = 0, 1, 2
NAMED_SCHEDULES = ("attn_only_1st_attn", "all_attn_25", "all_attn_35", "all_attn_50", "first_mamba", "second_mamba",
                   "all_attn_1m", "all_attn_2m", "sigmoid_25", "sigmoid_35", "sigmoid_50")


def schedule_step_decay(ranges: Sequence[Tuple[int, int, float]], L: int):
    """alpha_l from (lo, hi, alpha) ranges (inclusive, later ranges win; 1.0 elsewhere)."""
    n = len(ranges)
    lo = (ctypes.c_int * n)(*[int(r[0]) for r in ranges])
    hi = (ctypes.c_int * n)(*[int(r[1]) for r in ranges])
    al = (ctypes.c_double * n)(*[float(r[2]) for r in ranges])
    out = (ctypes.c_double * L)()
    _check(lib().strd_schedule_step_decay(ctypes.cast(lo, _vp), ctypes.cast(hi, _vp), ctypes.cast(al, _vp), n, int(L),
                                          ctypes.cast(out, _vp)), "schedule_step_decay")
    return list(out)


def hybrid_layout(L: int = HYBRID_LAYERS):
    """Layer types (LAYER_MAMBA / LAYER_MLP / LAYER_ATTN) of the 62-layer hybrid of the paper's schedules."""
    out = (ctypes.c_int32 * L)()
    _check(lib().strd_hybrid_layout(int(L), ctypes.cast(out, _vp)), "hybrid_layout")
    return list(out)


def schedule_named(name: str):
    """Retention ratios of one of NAMED_SCHEDULES for the 62 layers."""
    out = (ctypes.c_double * HYBRID_LAYERS)()
    _check(lib().strd_schedule_named(name.encode(), ctypes.cast(out, _vp)), "schedule_named(%s)" % name)
    return list(out)
