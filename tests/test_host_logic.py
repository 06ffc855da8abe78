"""CPU-only checks of the host side: the C ABI library loads and exports every symbol the
header declares, the schedule helpers reproduce the paper's printed arithmetic, and the input
generator is deterministic."""
import os
import re

import numpy as np
import pytest
import torch

import paper_2603_00198_amd as strd
from paper_2603_00198_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "strd.h")).read()
    declared = set(re.findall(r"\b(strd_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    L = strd.lib()
    for name in sorted(declared):
        assert hasattr(L, name), "libstrd.so does not export " + name
    assert declared == set(binding.exported_symbols())
    assert L.strd_version() >= 1000
    assert b"STRD_OK" in L.strd_status_string(0)


def _golden_schedules(golden_dir):
    rows = []
    for line in open(os.path.join(golden_dir, "schedule_step_decay.txt")):
        if line.strip() and not line.startswith("#"):
            name, comp, spec = line.split(None, 2)
            alpha = np.zeros(62)
            for part in spec.split(";"):
                rng, val = part.split("=")
                lo, hi = (int(v) for v in rng.split(":"))
                alpha[lo:hi + 1] = float(val)
            rows.append((name, float(comp), alpha))
    return rows


def test_step_decay_tables_reproduce_the_printed_compression(golden_dir):
    # App. "Reduction Schedule Configurations": Comp.% is the mean retention over the 62 layers,
    # with alpha relative to the original token count.
    N0 = 36864                                   # 256 frames x 144 tokens per frame
    for name, comp, alpha in _golden_schedules(golden_dir):
        K = strd.schedule_budgets(list(alpha), N0, K_min=144)
        assert len(K) == 62 and all(a >= b for a, b in zip(K, K[1:]))
        assert 100.0 * np.mean(K) / N0 == pytest.approx(comp, abs=0.06), name


def test_budgets_floor_clamp_and_monotone():
    assert strd.schedule_budgets([1, 1, .75, .75, .5, .5, .25, .25], 32768) == \
        [32768, 32768, 24576, 24576, 16384, 16384, 8192, 8192]
    assert strd.schedule_budgets([0.15], 36864) == [5529]           # floor(5529.6)
    assert strd.schedule_budgets([0.001, 0.5], 1000, K_min=144) == [144, 144]   # never grows back
    assert strd.schedule_budgets([0.5], 100, K_min=144) == [100]    # a single image is left whole
    with pytest.raises(strd.StrdError):
        strd.schedule_budgets([1.5], 10)


def test_sigmoid_schedule_shape():
    a = strd.schedule_sigmoid(62, 1.0, 0.125, 20.0, 0.24)
    assert a[0] == pytest.approx(0.125 + 0.875 / (1 + np.exp(-20 * 0.24)))
    assert all(x > y for x, y in zip(a, a[1:]))
    assert a[-1] == pytest.approx(0.125, abs=1e-4)
    mid = 0.24 * 62
    lo, hi = int(np.floor(mid)), int(np.ceil(mid))
    assert a[lo] >= (1.0 + 0.125) / 2 >= a[hi]


def test_named_schedules_match_the_printed_table(golden_dir):
    names = {"attn_only_1st_attn", "all_attn_25", "all_attn_35", "all_attn_50", "first_mamba"}
    seen = set()
    for name, comp, alpha in _golden_schedules(golden_dir):
        np.testing.assert_allclose(strd.schedule_named(name), alpha, rtol=0, atol=0)
        seen.add(name)
    assert seen == names
    second = strd.schedule_named("second_mamba")
    assert second[0] == 1.0 and set(second[1:]) == {0.23}
    assert strd.schedule_named("sigmoid_35") == strd.schedule_sigmoid(62, 1.0, 0.125, 20.0, 0.24)
    with pytest.raises(strd.StrdError):
        strd.schedule_named("no_such_schedule")


def test_step_decay_ranges_and_layout():
    assert strd.schedule_step_decay([(0, 1, 1.0), (2, 4, 0.5), (4, 4, 0.25)], 6) == [1.0, 1.0, 0.5, 0.5, 0.25, 1.0]
    with pytest.raises(strd.StrdError):
        strd.schedule_step_decay([(3, 9, 0.5)], 6)
    ty = strd.hybrid_layout()
    assert [l for l, t in enumerate(ty) if t == strd.LAYER_ATTN] == [7, 16, 25, 34, 43, 52]
    assert ty.count(strd.LAYER_MAMBA) == 28 and ty.count(strd.LAYER_MLP) == 28 and ty[0] == strd.LAYER_MAMBA


def test_interleaved_schedules_reduce_at_attention_and_the_mamba_layers_between():
    ty = strd.hybrid_layout()
    for name, per_gap in (("all_attn_1m", 1), ("all_attn_2m", 2)):
        a = strd.schedule_named(name)
        assert a[0] == 1.0 and all(x >= y for x, y in zip(a, a[1:]))
        drops = [l for l in range(1, 62) if a[l] < a[l - 1]]
        assert all(ty[l] != strd.LAYER_MLP for l in drops)
        assert a[drops[0]] == pytest.approx(0.32) and min(a) == pytest.approx(0.15)
        assert all(a[l] == pytest.approx(0.15) for l in range(34, 62))
        # every attention layer up to 33 reduces, and so do `per_gap` Mamba layers before each
        assert {7, 16, 25} <= set(drops)
        assert sum(ty[l] == strd.LAYER_MAMBA for l in drops if l < 7) == per_gap


def test_stack_model_adds_up():
    from paper_2603_00198_amd.stack import model_stack_time
    ty = strd.hybrid_layout()
    K = strd.schedule_budgets(strd.schedule_named("attn_only_1st_attn"), 1000)
    mix = lambda kind, n: float(n) if kind == "mamba" else float(n) ** 2 / 1000
    red, full = model_stack_time(ty, K, 1000, mix, lambda kind, n_in, k: 7.0)
    assert full == 28 * 1000 + 6 * 1000
    n_m_before = sum(t == strd.LAYER_MAMBA for t in ty[:7])
    assert red == pytest.approx(7.0 + n_m_before * 1000 + (28 - n_m_before) * 150 + 6 * 150 ** 2 / 1000)


def test_speedup_arithmetic_of_the_headline_claim(golden_dir):
    vals = {}
    for line in open(os.path.join(golden_dir, "ttft_25pct.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            vals[k] = float(v)
    ratios = [vals["baseline"] / v for k, v in vals.items() if k != "baseline"]
    assert min(ratios) == pytest.approx(3.8, abs=0.05) and max(ratios) == pytest.approx(4.2, abs=0.06)


def test_synthetic_inputs_are_seeded_and_shaped():
    w = synth.shrink(synth.WORKLOADS["c5"], N=1024, M=16, d_model=64)
    h1, h2 = synth.hidden_states(w), synth.hidden_states(w)
    assert torch.equal(h1, h2) and h1.shape == (1040, 64)
    t = synth.mamba_inputs(w, h1)
    assert t["x"].shape == (1040, 128, 64) and t["x"].dtype == torch.bfloat16
    assert t["B"].shape == (1040, 8, 128) and (t["dt"] > 0).all() and (t["A"] < 0).all()
    a = synth.attn_inputs(w, h1)
    assert a["q"].shape == (1040, 32, 128) and a["k"].shape == (1040, 8, 128)
    # outlier rows exist and frames share a component
    norms = h1[:1024].norm(dim=1)
    assert (norms > 4 * norms.median()).float().mean() > 0.02
    assert synth.WORKLOADS["c2"].K == 2048 and synth.WORKLOADS["c3"].K == 8192


def test_kernels_with_split_lds_reads_do_not_spill():
    """ssd_mfma.hip, ssd_seg_mfma.hip, attn_mfma.hip and linear_mfma.hip issue LDS reads from inline assembly and wait for them later;
    between the two the compiler believes the destination registers hold their values.  A spill of
    such a register before the wait would save garbage, so these kernels must fit their register
    budget without scratch memory.  The compiler's own resource report is the check."""
    import subprocess
    from paper_2603_00198_amd import build as strd_build
    for name in ("ssd_mfma.hip", "ssd_seg_mfma.hip", "attn_mfma.hip", "linear_mfma.hip"):
        src = os.path.join(strd_build.CSRC, name)
        cmd = [strd_build.HIPCC] + strd_build.FLAGS + ["--cuda-device-only", "-c", src, "-o", os.devnull,
                                                       "-Rpass-analysis=kernel-resource-usage"]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        scratch = [int(v) for v in re.findall(r"ScratchSize \[bytes/lane\]: (\d+)", r.stderr)]
        assert scratch, "no resource report for " + name
        assert all(v == 0 for v in scratch), "%s: a kernel uses scratch memory: %s" % (name, scratch)
        # a register saved to another register file (no scratch needed) would carry stale data just the same
        for what in ("VGPRs Spill", "SGPRs Spill", "AGPRs"):
            vals = [int(v) for v in re.findall(what + r": (\d+)", r.stderr)]
            assert len(vals) == len(scratch) and all(v == 0 for v in vals), "%s: %s = %s" % (name, what, vals)


def test_entry_points_refuse_inconsistent_arguments_on_the_host():
    """Every compute entry point validates its arguments on the host and returns STRD_EINVAL before
    anything is launched: one field at a time is made inconsistent in an otherwise consistent call.
    The pointers are placeholders that are never dereferenced on the host, which is why this runs only
    where no GPU is visible (a call that slipped through validation then ends in a HIP error code,
    not in a launch)."""
    if torch.cuda.is_available():
        pytest.skip("placeholder pointers: only run without a GPU")
    L = binding.lib()
    P, BIG, F32, BF16 = 0x1000, 1 << 40, 0, 1
    EINVAL, EHIP = -1, -4
    # name -> (consistent argument list, {position: inconsistent value, ...})
    cases = {
        "strd_score_attn": ([P, P, P, 8, 100, 4, 2, 64, 0.125, BF16, P, BIG, None],
                            {0: None, 1: None, 2: None, 3: 0, 4: 0, 5: 3, 6: 0, 7: 0, 8: 0.0, 9: 7}),
        "strd_score_mamba": ([P, P, P, P, 8, 100, 8, 2, 64, BF16, P, BIG, None],
                             {0: None, 1: None, 2: None, 3: None, 4: 0, 5: 0, 6: 7, 7: 0, 8: 0, 9: 7}),
        "strd_score_mamba_full": ([P, P, P, P, P, 8, 100, 8, 2, 64, BF16, P, BIG, None],
                                  {0: None, 2: None, 3: None, 4: None, 5: 0, 6: 0, 7: 7, 8: 0, 9: 0, 10: 7}),
        "strd_select_topk": ([P, 100, 10, P, None, 0, None], {0: None, 1: 0, 2: 0, 3: None}),
        "strd_select_topk_noalloc": ([P, 100, 10, P, None], {0: None, 1: 0, 2: 0, 3: None}),
        "strd_compact": ([P, P, P, 100, 4, 10, 64, None, None, None], {1: None, 2: None, 3: -1, 4: -1, 5: 101, 6: 6}),
        "strd_ssd_prefill": ([P, P, P, P, P, None, None, P, None, 64, 8, 64, 2, 128, 64, BF16, P, BIG, None],
                             {0: None, 1: None, 2: None, 3: None, 4: None, 7: None, 9: -1, 10: 7, 11: 0, 12: 0, 13: 0,
                              14: 0, 15: 7}),
        "strd_ssd_prefill_gather": ([P, P, P, P, P, None, None, P, P, None, 100, 4, 10, 8, 64, 2, 128, 64, BF16, None, 0, None],
                                    {0: None, 2: None, 7: None, 8: None, 10: -1, 11: -1, 12: 101, 13: 7, 14: 0, 16: 0,
                                     17: 0, 18: 7}),
        "strd_attn_prefill": ([P, P, P, P, 64, 4, 2, 128, 0.09, BF16, P, BIG, None],
                              {0: None, 1: None, 2: None, 3: None, 4: -1, 5: 3, 6: 0, 7: 0, 8: -1.0, 9: 7}),
        "strd_rmsnorm": ([P, P, P, 8, 64, 1e-5, BF16, None], {0: None, 1: None, 2: None, 3: -1, 4: 0, 5: -1.0, 6: 7}),
        "strd_avgpool": ([P, P, 100, 4, 10, 64, BF16, None, None, None], {1: None, 2: -1, 3: -1, 4: 101, 6: 7}),
        "strd_linear_mfma": ([P, P, None, P, 100, 128, 264, BF16, None], {0: None, 1: None, 3: None, 4: -1, 5: 0, 6: 0, 7: 7}),
        "strd_linear": ([P, P, None, P, 4352, 256, 4096, BF16, None], {0: None, 1: None, 3: None, 4: -1, 5: 0, 6: 0, 7: 7}),
        "strd_attn_decode_step": ([P, P, P, P, 100, 4, 2, 64, 0.125, BF16, P, BIG, None], {0: None, 3: None, 4: 0, 5: 3, 9: 7}),
    }
    for name, (good, bad) in cases.items():
        fn = getattr(L, name)
        assert len(good) == len(fn.argtypes), name
        # the consistent call gets past validation and, with no GPU, fails loudly: a HIP error code, no fallback
        assert fn(*good) == EHIP, name
        for pos, value in bad.items():
            args = list(good)
            args[pos] = value
            rc = fn(*args)
            assert rc == EINVAL, "%s accepted argument %d = %r (returned %d)" % (name, pos, value, rc)


def test_rate_probe_refuses_empty_launches():
    L = binding.lib()
    assert L.strd_mfma_rate_probe(None, 4, 10, 0, None) == -1
    assert L.strd_mfma_rate_probe(0x1000, 0, 10, 0, None) == -1
    assert L.strd_mfma_rate_probe(0x1000, 4, 0, 1, None) == -1
    assert L.strd_mfma_rate_probe(0x1000, 4, 10, 4, None) == -1


def test_packed_batch_entry_points_validate_their_descriptors_on_the_host():
    """The sequence descriptors of the *_varlen calls are a host array: counts, K <= N, the score
    row length and the limit on sequences per call are checked before anything is launched."""
    if torch.cuda.is_available():
        pytest.skip("placeholder pointers: only run without a GPU")
    import ctypes
    L = binding.lib()
    P, BIG, BF16 = 0x1000, 1 << 40, 1
    EINVAL, EUNSUPPORTED, EHIP = -1, -2, -4

    def seqs(*t):
        arr = (binding._Seq * len(t))()
        for i, (n, m, k) in enumerate(t):
            arr[i].N, arr[i].M, arr[i].K = n, m, k
        return ctypes.cast(arr, ctypes.c_void_p), len(t), arr

    good, ng, keep = seqs((100, 8, 10), (37, 3, 37))
    mamba = lambda sq, nsq, ld=100: L.strd_score_mamba_varlen(P, P, P, P, ld, sq, nsq, 8, 2, 64, BF16, P, BIG, None)
    attn = lambda sq, nsq, ld=100: L.strd_score_attn_varlen(P, P, P, ld, sq, nsq, 4, 2, 64, 0.125, BF16, P, BIG, None)
    topk = lambda sq, nsq, ld=100: L.strd_select_topk_varlen(P, ld, sq, nsq, P, None)
    item = (binding._CompactItem * 1)()
    item[0].src, item[0].dst, item[0].row_bytes = P, P, 64
    comp = lambda sq, nsq: L.strd_compact_varlen(ctypes.cast(item, ctypes.c_void_p), 1, P, sq, nsq, None, None, None)
    for call in (mamba, attn, topk, comp):
        assert call(good, ng) == EHIP            # consistent: past validation, then no GPU
        assert call(None, ng) == EINVAL
        assert call(good, 0) == EINVAL
        assert call(good, 65) == EINVAL          # STRD_VARLEN_MAX sequences per call
        for bad in ((0, 8, 1), (100, 0, 10)):
            sq, nsq, k2 = seqs((100, 8, 10), bad)
            assert call(sq, nsq) == EINVAL, bad
    for call in (mamba, attn, topk):
        assert call(good, ng, 96) == EINVAL      # shorter than the longest sequence
        assert call(good, ng, 102) == EINVAL     # not a multiple of 4
    for bad in ((100, 8, 0), (100, 8, 101)):     # K is checked where it is used ...
        sq, nsq, k2 = seqs(bad)
        assert topk(sq, nsq) == EINVAL and comp(sq, nsq) == EINVAL
        assert mamba(sq, nsq) == EHIP and attn(sq, nsq) == EHIP  # ... and ignored by the scores
    sq, nsq, k2 = seqs((40000, 8, 10))
    assert topk(sq, nsq, 40000) == EUNSUPPORTED   # one workgroup per sequence: at most 32768 scores each
    assert L.strd_select_topk_varlen_max_n() == 32768
    assert L.strd_score_mamba_varlen_workspace(good, ng, 8, 2, 64, BF16) >= (100 + 8 + 37 + 3) * 2 * 4
    assert L.strd_score_mamba_varlen_workspace(good, ng, 8, 2, 40, BF16) == 0
    assert L.strd_score_attn_varlen_workspace(good, ng, 4, 2, 64, BF16) > 0


def test_matrix_core_shapes_refuse_misaligned_tensors_and_report_their_kernel_path():
    """16-byte vectors are moved straight from the caller's pointers on the matrix-core shapes: a
    misaligned tensor is refused on the host.  Which kernel a shape runs is answered without a GPU."""
    L = binding.lib()
    P, BIG, F32, BF16 = 0x1000, 1 << 40, 0, 1
    EINVAL = -1
    assert L.strd_score_attn(P + 8, P, P, 8, 100, 4, 2, 64, 0.125, BF16, P, BIG, None) == EINVAL
    assert L.strd_score_mamba(P, P + 2, P, P, 8, 100, 8, 2, 64, BF16, P, BIG, None) == EINVAL
    assert L.strd_ssd_prefill(P + 4, P, P, P, P, None, None, P, None, 64, 8, 64, 2, 128, 64, BF16, P, BIG, None) == EINVAL
    assert L.strd_attn_prefill(P, P, P + 8, P, 64, 4, 2, 128, 0.09, BF16, P, BIG, None) == EINVAL
    assert L.strd_select_topk(P + 4, 100, 10, P, None, 0, None) == EINVAL
    assert L.strd_select_topk_noalloc(P + 4, 100, 10, P, None) == EINVAL
    # the library's own projection kernel: misaligned tensors, and the shapes it is not tiled for
    EUNSUPPORTED = -2
    assert L.strd_linear_mfma(P + 8, P, None, P, 100, 128, 264, BF16, None) == EINVAL
    assert L.strd_linear_mfma(P, P, P + 2, P, 100, 128, 264, BF16, None) == EINVAL
    assert L.strd_linear_mfma(P, P, None, P, 100, 100, 264, BF16, None) == EUNSUPPORTED   # Kd not a multiple of 64
    assert L.strd_linear_mfma(P, P, None, P, 100, 128, 100, BF16, None) == EUNSUPPORTED   # Nd not a multiple of 8
    assert L.strd_linear_mfma(P, P, None, P, 100, 128, 264, F32, None) == EUNSUPPORTED    # bf16 only
    assert L.strd_linear_mfma(P, P, None, P, 0, 128, 264, BF16, None) == 0                # nothing to do
    assert L.strd_linear_mfma_supported(33024, 4096, 18560, BF16) == 1
    assert L.strd_linear_mfma_supported(1 << 20, 4096, 8, BF16) == 0                      # x of 8 GiB: 32-bit copy offsets
    kp = strd.kernel_path
    bf, f32 = torch.bfloat16, torch.float32
    assert kp("score_attn", 256, 32768, 32, 8, 128) == strd.PATH_MFMA
    assert kp("score_attn", 256, 32768, 32, 8, 96) == strd.PATH_SIMT
    assert kp("score_attn", 32, 1024, 4, 2, 64, dtype=f32) == strd.PATH_SIMT
    assert kp("score_attn", 32, 1024, 4, 3, 64) == strd.PATH_NONE
    assert kp("score_mamba", 128, 8192, 128, 8, 128) == strd.PATH_MFMA
    assert kp("score_mamba", 128, 8192, 128, 8, 40) == strd.PATH_SIMT
    assert kp("ssd_prefill", 2176, 128, 64, 8, 128) == strd.PATH_MFMA
    assert kp("ssd_prefill", 2176, 128, 24, 8, 128) == strd.PATH_SIMT
    assert kp("ssd_prefill", 1056, 8, 32, 1, 16, dtype=f32) == strd.PATH_SIMT
    assert kp("attn_prefill", 8448, 32, 8, 128) == strd.PATH_MFMA
    assert kp("attn_prefill", 100, 6, 3, 40) == strd.PATH_SIMT
    assert kp("attn_prefill", 100, 6, 4, 64) == strd.PATH_NONE
