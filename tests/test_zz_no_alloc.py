"""The selection entry point that allocates nothing (its scratch is an array inside the library's
image) against the ordinary one, through the C ABI, on two calls in a row, the second smaller.
Needs a GPU.  Collected last: a failure here must not hide the tests before it."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2603_00198_amd as strd

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _both(L, scores, K):
    """idx from strd_select_topk (caller's workspace) and from strd_select_topk_noalloc, raw C calls."""
    N = scores.shape[0]
    stream = torch.cuda.current_stream().cuda_stream
    want = torch.full((K,), -1, dtype=torch.int32, device=DEV)
    got = torch.full((K,), -1, dtype=torch.int32, device=DEV)
    need = L.strd_select_topk_workspace(N, K)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=DEV)
    assert L.strd_select_topk(scores.data_ptr(), N, K, want.data_ptr(), ws.data_ptr(), ws.numel(), stream) == 0
    assert L.strd_select_topk_noalloc(scores.data_ptr(), N, K, got.data_ptr(), stream) == 0
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


def test_select_topk_noalloc_matches_select_topk_on_two_calls_in_a_row():
    L = strd.lib()
    assert L.strd_select_topk_noalloc_max_n() == 1 << 20
    r = np.random.default_rng(5)
    # both sizes take the many-workgroup form, i.e. the one that uses the scratch array; the second
    # call is smaller and finds the first call's histograms and counts in it
    for N, K in ((200003, 65536), (40000, 1234), (131072, 32768), (33000, 32999)):
        print("[case] select_topk_noalloc N=%d K=%d" % (N, K), flush=True)
        s_np = (r.random(N, dtype=np.float32) ** 3).astype(np.float32)
        s_np[::53] = s_np[7]                                  # ties across tiles
        scores = torch.from_numpy(s_np).to(DEV)
        got, want = _both(L, scores, K)
        np.testing.assert_array_equal(got, want)
        np.testing.assert_array_equal(got, oracle.select_topk(s_np.astype(np.float64), K))
    # one-workgroup sizes never touch the array; they must still agree
    for N, K in ((8192, 2048), (5, 3)):
        print("[case] select_topk_noalloc N=%d K=%d" % (N, K), flush=True)
        scores = torch.from_numpy(r.random(N, dtype=np.float32)).to(DEV)
        got, want = _both(L, scores, K)
        np.testing.assert_array_equal(got, want)


def test_select_topk_noalloc_refuses_what_does_not_fit():
    L = strd.lib()
    N = (1 << 20) + 1
    scores = torch.rand(N, device=DEV)
    idx = torch.full((8,), -7, dtype=torch.int32, device=DEV)
    stream = torch.cuda.current_stream().cuda_stream
    assert L.strd_select_topk_noalloc(scores.data_ptr(), N, 8, idx.data_ptr(), stream) == -2      # STRD_EUNSUPPORTED
    assert L.strd_select_topk_noalloc(scores.data_ptr(), 100, 0, idx.data_ptr(), stream) == -1    # STRD_EINVAL
    assert L.strd_select_topk_noalloc(None, 100, 8, idx.data_ptr(), stream) == -1
    torch.cuda.synchronize()
    assert (idx.cpu().numpy() == -7).all()                   # nothing was launched
    out = strd.select_topk_noalloc(scores[:50000].contiguous(), 8, idx)                              # the binding, too
    np.testing.assert_array_equal(out.cpu().numpy(), strd.select_topk(scores[:50000].contiguous(), 8).cpu().numpy())
