"""GPU parity of the variants around the reduced prefill: the average-pool reduction baseline and
the single-token decode steps that take over the state and the cache a reduced prefill leaves."""
import numpy as np
import pytest
import torch

import oracle
import paper_2603_00198_amd as strd
from paper_2603_00198_amd import synth
from util import TOL, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print("[case] " + msg, flush=True)


# ------------------------------------------------------------------ avgpool ----------------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("N,M,K,D", [
    (1024, 32, 256, 256),    # ratio 4, vector path
    (1000, 7, 333, 136),     # ragged windows of 3 and 4 rows
    (513, 0, 100, 64),       # windows of 5 and 6 rows: more than one trip of the 4-row batches
    (300, 5, 300, 8),        # K = N: identity
    (77, 3, 1, 24),          # one window over everything
    (90, 4, 13, 7),          # 7 columns: scalar path
    (0, 6, 0, 16),           # no vision tokens
])
def test_avgpool_parity(N, M, K, D, dtype):
    _say("avgpool N=%d M=%d K=%d D=%d %s" % (N, M, K, D, dtype))
    g = torch.Generator().manual_seed(N + K + D)
    src = torch.randn(N + M, D, generator=g).to(dtype)
    pos_in = torch.randperm(7 * (N + M), generator=g)[: N + M].to(torch.int32)
    dst, pos = strd.avgpool(src.to(DEV), N, M, K, pos_in=pos_in.to(DEV))
    want, want_pos = oracle.avgpool(synth.np64(src), N, M, K, pos_in.numpy())
    np.testing.assert_array_equal(pos.cpu().numpy(), want_pos)
    assert dst.shape == (K + M, D)
    if K + M:
        assert_close(synth.np64(dst), want, TOL[dtype], "avgpool")
        # the text tail is a copy, bit for bit
        assert torch.equal(dst[K:].cpu(), src[N:])
    _, pos_id = strd.avgpool(src.to(DEV), N, M, K, want_pos=True)
    np.testing.assert_array_equal(pos_id.cpu().numpy(), oracle.avgpool(synth.np64(src), N, M, K)[1])


def test_avgpool_errors():
    x = torch.zeros(10, 8, device=DEV)
    with pytest.raises(strd.StrdError):
        strd.avgpool(x, 8, 2, 9)        # K > N
    with pytest.raises(strd.StrdError):
        strd.avgpool(x, 8, 2, 0)        # vision rows but no window
    with pytest.raises(strd.StrdError):
        strd.avgpool(x, 7, 2, 3)        # rows do not add up


# ------------------------------------------------------------------ ssd_decode_step --------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("H,P,G,n,with_D", [
    (8, 64, 2, 128, True),     # lanes = 32, the paper's state width
    (6, 32, 3, 64, False),     # lanes = 16
    (4, 5, 1, 16, True),       # narrow state, rows do not fill the last workgroup
    (3, 7, 3, 10, True),       # n not a multiple of 4: scalar columns
    (2, 3, 1, 200, False),     # wider than one trip of the lanes
])
def test_ssd_decode_step_parity(H, P, G, n, with_D, dtype):
    _say("ssd_decode_step H=%d P=%d G=%d n=%d D=%s %s" % (H, P, G, n, with_D, dtype))
    g = torch.Generator().manual_seed(H * P + n)
    x = torch.randn(H, P, generator=g).to(dtype)
    dt = torch.nn.functional.softplus(torch.randn(H, generator=g))
    A = -torch.exp(2 * torch.rand(H, generator=g))
    B = torch.randn(G, n, generator=g).to(dtype)
    C = torch.randn(G, n, generator=g).to(dtype)
    D = torch.randn(H, generator=g) if with_D else None
    S = torch.randn(H, P, n, generator=g)
    S_dev = S.to(DEV)
    y = strd.ssd_decode_step(x.to(DEV), dt.to(DEV), A.to(DEV), B.to(DEV), C.to(DEV),
                             None if D is None else D.to(DEV), S_dev)
    y_ref, S_ref = oracle.ssd_decode_step(synth.np64(x), synth.np64(dt), synth.np64(A), synth.np64(B), synth.np64(C),
                                          None if D is None else synth.np64(D), synth.np64(S))
    assert_close(synth.np64(S_dev), S_ref, 1e-5, "state")          # the state stays fp32 for either io dtype
    assert_close(synth.np64(y), y_ref, TOL[dtype], "y", units=(0,))


def test_decode_continues_a_reduced_mamba_prefill():
    """Reduced prefill (score, top-K, gather-fused scan) -> S_out -> two decode steps, against the
    oracle run over the retained tokens followed by the two new tokens."""
    _say("reduced prefill then decode, Mamba-2")
    N, M, K = 600, 40, 150
    w = synth.Workload("decode-m", N=N, M=M + 2, d_model=256, dtype="bf16",   # the last two rows are the new tokens
                       mamba=synth.MambaShape(H=8, P=64, n=128, G=2, chunk=64), seed=3)
    dev = synth.mamba_inputs(w, synth.hidden_states(w, DEV))
    t = dev
    T0 = N + M
    scores = strd.score_mamba(dev["B"][:N], dev["C"][N:T0], dev["dt"][:N])
    idx = strd.select_topk(scores, K)
    y, S = strd.ssd_prefill_gather(dev["x"][:T0], dev["dt"][:T0], dev["A"], dev["B"][:T0], dev["C"][:T0], idx, N, M)
    ys = []
    for j in (T0, T0 + 1):
        ys.append(strd.ssd_decode_step(dev["x"][j], dev["dt"][j], dev["A"], dev["B"][j], dev["C"][j], None, S))
    keep = np.r_[idx.cpu().numpy(), np.arange(N, T0 + 2)]
    n64 = {k: synth.np64(v) for k, v in t.items()}
    y_ref, S_ref = oracle.ssd_seq(n64["x"][keep], n64["dt"][keep], n64["A"], n64["B"][keep], n64["C"][keep])
    assert_close(synth.np64(torch.stack(ys)), y_ref[-2:], TOL[torch.bfloat16], "decoded y", units=(0, 1))
    assert_close(synth.np64(S), S_ref, TOL[torch.bfloat16], "state after decode", units=(0,))


# ------------------------------------------------------------------ attn_decode_step -------
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,Hq,Hkv,d", [
    (1, 4, 2, 64),          # only the token itself
    (63, 8, 2, 128),        # one ragged slice, 4 query heads per kv head
    (200, 8, 8, 64),        # several slices, ragged tail, one query head per kv head
    (1000, 16, 2, 128),     # 8 query heads per kv head
    (17000, 4, 2, 64),      # several trips per wave, odd number of trips
    (70000, 4, 2, 64),      # long cache: 256-token slices
])
def test_attn_decode_step_parity(T, Hq, Hkv, d, dtype):
    _say("attn_decode_step T=%d Hq=%d Hkv=%d d=%d %s" % (T, Hq, Hkv, d, dtype))
    g = torch.Generator().manual_seed(T + Hq + d)
    q = torch.randn(Hq, d, generator=g).to(dtype)
    k = torch.randn(T, Hkv, d, generator=g).to(dtype)
    v = torch.randn(T, Hkv, d, generator=g).to(dtype)
    if T > 100:                                  # one key the query clearly prefers: a peaked row
        k[T // 3] = (3 * q.float().view(Hkv, Hq // Hkv, d).mean(1)).to(dtype)
    o = strd.attn_decode_step(q.to(DEV), k.to(DEV), v.to(DEV))
    ref = oracle.attn_decode_step(synth.np64(q), synth.np64(k), synth.np64(v))
    assert_close(synth.np64(o), ref, TOL[dtype], "attn_decode_step", units=(0,))


def test_decode_continues_a_reduced_attention_prefill():
    """The last row of a prefill over the K + M survivors plus one new token equals the decode step
    over the compacted cache."""
    _say("reduced prefill then decode, attention")
    N, M, K = 500, 30, 120
    w = synth.Workload("decode-a", N=N, M=M + 1, d_model=256, dtype="bf16",   # the last row is the new token
                       attn=synth.AttnShape(Hq=8, Hkv=2, d=128), seed=4)
    dev = synth.attn_inputs(w, synth.hidden_states(w, DEV))
    t = dev
    T0 = N + M
    scores = strd.score_attn(dev["q"][N:T0], dev["k"][:N])
    idx = strd.select_topk(scores, K)
    (kc, vc), _ = strd.compact_batch([dev["k"][:T0], dev["v"][:T0]], idx, N, M)
    k_cache = torch.cat([kc, dev["k"][T0:T0 + 1]])          # the new token's row is appended by the caller
    v_cache = torch.cat([vc, dev["v"][T0:T0 + 1]])
    o = strd.attn_decode_step(dev["q"][T0], k_cache, v_cache)
    keep = np.r_[idx.cpu().numpy(), np.arange(N, T0 + 1)]
    n64 = {k: synth.np64(v) for k, v in t.items()}
    ref = oracle.attn(n64["q"][keep], n64["k"][keep], n64["v"][keep], rows=[K + M])[0]
    assert_close(synth.np64(o), ref, TOL[torch.bfloat16], "decode over the compacted cache", units=(0,))
    # and it agrees with the prefill kernel run over the same K + M + 1 rows
    o_pre = strd.attn_prefill(dev["q"][torch.from_numpy(keep).to(DEV)].contiguous(), k_cache, v_cache)[-1]
    assert_close(synth.np64(o), synth.np64(o_pre), TOL[torch.bfloat16], "decode vs prefill last row")


def test_attn_decode_step_errors():
    q = torch.zeros(6, 64, device=DEV)
    kv = torch.zeros(10, 2, 64, device=DEV)
    with pytest.raises(strd.StrdError):
        strd.attn_decode_step(q, kv, kv)                       # 3 query heads per kv head: unsupported
    q = torch.zeros(4, 32, device=DEV)
    kv = torch.zeros(10, 2, 32, device=DEV)
    with pytest.raises(strd.StrdError):
        strd.attn_decode_step(q, kv, kv)                       # d = 32: unsupported


def test_matrix_core_rate_probe_counts_its_products():
    """The measurement aid of the benchmark: with every operand 1.0 each of the 64 accumulator entries
    of a lane ends at iters * 8 products * 16 = iters * 128, so the lane's checksum is iters * 8192."""
    out = strd.mfma_rate_probe(8, 50, False)
    assert out.shape == (8 * 256,) and bool((out == 50 * 8192).all())
    rnd = strd.mfma_rate_probe(8, 50, True)
    assert bool(torch.isfinite(rnd).all()) and float(rnd.abs().max()) > 0
    # the 16 x 16 x 32 form: 32 accumulator entries per lane, each iters * 8 products * 32
    small = strd.mfma_rate_probe(8, 50, False, small_products=True)
    assert bool((small == 50 * 8192).all())
