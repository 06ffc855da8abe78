"""Seeded synthetic inputs shaped like the paper's long-video workloads.

This module holds input generation only -- none of the method's arithmetic --
so that the tests can hand identical tensors to the HIP library and to the CPU
oracle.  A sequence is N vision tokens (frames x tokens-per-frame) followed by
M text tokens (paper Sec. 3.1).  Hidden states are Gaussian; the mixer inputs
are seeded Gaussian projections of them (set-up glue, outside the library);
dt = softplus(N(0,1)) > 0 and A = -exp(U(0,2)) < 0 per head.  All random numbers come from
torch's CPU generator, once, in fp32, whatever device the tensors then live on; the projections
(fp32 matrix products, set-up only) run where the tensors are.

The real workloads (long-video benchmarks at 256-512 frames) are not
available offline; these tensors stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import torch


@dataclass(frozen=True)
class MambaShape:
    H: int       # heads
    P: int       # head dim
    n: int       # state dim
    G: int       # B/C groups
    chunk: int


@dataclass(frozen=True)
class AttnShape:
    Hq: int
    Hkv: int
    d: int


@dataclass(frozen=True)
class Workload:
    name: str
    N: int                      # vision tokens
    M: int                      # text tokens (last)
    d_model: int
    dtype: str                  # "f32" | "bf16"
    mamba: Optional[MambaShape] = None
    attn: Optional[AttnShape] = None
    budget: float = 0.25
    tokens_per_frame: int = 256
    frame_corr: float = 0.0     # rho of the per-frame shared component
    outlier_frac: float = 0.0   # fraction of vision tokens scaled by outlier_scale
    outlier_scale: float = 8.0
    seed: int = 0

    @property
    def T(self) -> int:
        return self.N + self.M

    @property
    def K(self) -> int:
        return int(self.budget * self.N)


_BIG_MAMBA = MambaShape(H=128, P=64, n=128, G=8, chunk=256)
_BIG_ATTN = AttnShape(Hq=32, Hkv=8, d=128)

WORKLOADS: Dict[str, Workload] = {
    # tiny fp32 pair
    "c1": Workload("c1", N=1024, M=32, d_model=256, dtype="f32",
                   mamba=MambaShape(H=8, P=32, n=16, G=1, chunk=64),
                   attn=AttnShape(Hq=4, Hkv=2, d=64), budget=0.5),
    # single Mamba-2 layer, 32 frames x 256
    "c2": Workload("c2", N=8192, M=128, d_model=4096, dtype="bf16", mamba=_BIG_MAMBA),
    # single attention layer, 128 frames x 256
    "c3": Workload("c3", N=32768, M=256, d_model=4096, dtype="bf16", attn=_BIG_ATTN),
    # 8-layer hybrid stack shapes
    "c4": Workload("c4", N=32768, M=256, d_model=4096, dtype="bf16", mamba=_BIG_MAMBA, attn=_BIG_ATTN),
    # long video, 512 frames x 256, correlated frames + outliers
    "c5": Workload("c5", N=131072, M=512, d_model=4096, dtype="bf16", mamba=_BIG_MAMBA,
                   attn=_BIG_ATTN, frame_corr=0.7, outlier_frac=0.05),
}

# retention ratio per layer of the 8-layer stack (6 Mamba-2 + 2 attention); the layers that
# reduce are 2 and 4 (Mamba-2) and 6 (attention), so both scores are used inside the stack
C4_RETAIN = (1.0, 1.0, 0.75, 0.75, 0.5, 0.5, 0.25, 0.25)
C4_LAYERS = ("mamba", "mamba", "mamba", "attn", "mamba", "mamba", "attn", "mamba")


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _gen(seed: int, device=None) -> torch.Generator:
    """Every random number is drawn on the host (torch's CPU generator), whatever device the tensor
    is for: a workload is the same tensor on every box.  `device` is accepted for the callers' sake."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def _randn(g: torch.Generator, device, *shape) -> torch.Tensor:
    return torch.randn(*shape, generator=g, dtype=torch.float32).to(device)


def _rand(g: torch.Generator, device, *shape) -> torch.Tensor:
    return torch.rand(*shape, generator=g, dtype=torch.float32).to(device)


def hidden_states(w: Workload, device="cpu", seed: Optional[int] = None) -> torch.Tensor:
    """[N+M, d_model] fp32 hidden states (vision rows first)."""
    g = _gen(w.seed if seed is None else seed, device)
    h = _randn(g, device, w.T, w.d_model)
    if w.frame_corr > 0.0:
        nf = (w.N + w.tokens_per_frame - 1) // w.tokens_per_frame
        f = _randn(g, device, nf, w.d_model)
        rho = w.frame_corr
        shared = f.repeat_interleave(w.tokens_per_frame, dim=0)[: w.N]
        h[: w.N] = rho * shared + (1.0 - rho * rho) ** 0.5 * h[: w.N]
    if w.outlier_frac > 0.0:
        pick = _rand(g, device, w.N) < w.outlier_frac
        h[: w.N][pick] *= w.outlier_scale
    return h


def _project(h: torch.Tensor, out_features: int, g: torch.Generator, rows: int = 16384) -> torch.Tensor:
    wgt = _randn(g, h.device, h.shape[1], out_features)
    wgt /= h.shape[1] ** 0.5
    out = torch.empty(h.shape[0], out_features, device=h.device, dtype=torch.float32)
    for r0 in range(0, h.shape[0], rows):
        out[r0:r0 + rows] = h[r0:r0 + rows] @ wgt
    return out


def mamba_inputs(w: Workload, hidden: torch.Tensor, seed: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """x [T,H,P], B,C [T,G,n] in the workload dtype; dt [T,H], A [H] fp32."""
    s = w.mamba
    dev = hidden.device
    g = _gen((w.seed if seed is None else seed) + 1001, dev)
    dt_io = torch_dtype(w.dtype)
    T = hidden.shape[0]
    x = _project(hidden, s.H * s.P, g).to(dt_io).view(T, s.H, s.P)
    B = _project(hidden, s.G * s.n, g).to(dt_io).view(T, s.G, s.n)
    C = _project(hidden, s.G * s.n, g).to(dt_io).view(T, s.G, s.n)
    dt = torch.nn.functional.softplus(_randn(g, dev, T, s.H))
    A = -torch.exp(2.0 * _rand(g, dev, s.H))
    return {"x": x.contiguous(), "B": B.contiguous(), "C": C.contiguous(), "dt": dt.contiguous(), "A": A}


def attn_inputs(w: Workload, hidden: torch.Tensor, seed: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """q [T,Hq,d], k,v [T,Hkv,d] in the workload dtype."""
    s = w.attn
    dev = hidden.device
    g = _gen((w.seed if seed is None else seed) + 2002, dev)
    dt_io = torch_dtype(w.dtype)
    T = hidden.shape[0]
    q = _project(hidden, s.Hq * s.d, g).to(dt_io).view(T, s.Hq, s.d)
    k = _project(hidden, s.Hkv * s.d, g).to(dt_io).view(T, s.Hkv, s.d)
    v = _project(hidden, s.Hkv * s.d, g).to(dt_io).view(T, s.Hkv, s.d)
    return {"q": q.contiguous(), "k": k.contiguous(), "v": v.contiguous()}


CONV_WIDTH = 4   # taps of the short causal convolution of a Mamba-2 block


def mamba_block_weights(w: Workload, device="cpu", seed: int = 0) -> Dict[str, torch.Tensor]:
    """Random-init weights of one Mamba-2 block at the workload's shapes (set-up only).  Matrices
    are [in, out] for y = x . W; scales keep activations O(1)."""
    s = w.mamba
    g = _gen(1000 + seed, device)
    dt_ = torch_dtype(w.dtype)
    d_inner, gn = s.H * s.P, s.G * s.n
    rn = lambda *shape: _randn(g, device, *shape)
    return {
        "norm_w": (1.0 + 0.1 * rn(w.d_model)).to(dt_),
        "W_z": (rn(w.d_model, d_inner) / w.d_model ** 0.5).to(dt_),
        "W_xbcdt": (rn(w.d_model, d_inner + 2 * gn + s.H) / w.d_model ** 0.5).to(dt_),
        "conv_w": (rn(d_inner + 2 * gn, CONV_WIDTH) / CONV_WIDTH ** 0.5).to(dt_),
        "conv_b": (0.1 * rn(d_inner + 2 * gn)).to(dt_),
        "dt_bias": rn(s.H).float(),
        "A": -torch.exp(2.0 * _rand(g, device, s.H)).float(),
        "D": rn(s.H).float(),
        "gnorm_w": (1.0 + 0.1 * rn(d_inner)).to(dt_),
        "W_out": (rn(d_inner, w.d_model) / d_inner ** 0.5).to(dt_),
    }


def attn_block_weights(w: Workload, device="cpu", seed: int = 0) -> Dict[str, torch.Tensor]:
    """Random-init weights of one attention block (no positional encoding) at the workload's shapes."""
    s = w.attn
    g = _gen(2000 + seed, device)
    dt_ = torch_dtype(w.dtype)
    rn = lambda *shape: _randn(g, device, *shape)
    return {
        "norm_w": (1.0 + 0.1 * rn(w.d_model)).to(dt_),
        "W_q": (rn(w.d_model, s.Hq * s.d) / w.d_model ** 0.5).to(dt_),
        "W_k": (rn(w.d_model, s.Hkv * s.d) / w.d_model ** 0.5).to(dt_),
        "W_v": (rn(w.d_model, s.Hkv * s.d) / w.d_model ** 0.5).to(dt_),
        "W_o": (rn(s.Hq * s.d, w.d_model) / (s.Hq * s.d) ** 0.5).to(dt_),
    }


def shrink(w: Workload, N: int, M: int, **kw) -> Workload:
    """Same layer shapes on a shorter sequence (parity cases the oracle finishes in seconds)."""
    from dataclasses import replace
    return replace(w, N=N, M=M, **kw)


def np64(t: torch.Tensor):
    """Exact up-conversion of a tensor to a float64 numpy array (for the oracle side of a test)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
