"""GPU parity of calibrations that hold more columns than one forward pass (16): consecutive passes of equal column
counts run together, the weight kernels serving both from one read of the weights.  Every case is compared with the
oracle, sequence by sequence, and with the same calibration run one pass at a time (EASYSPEC_PAIR_PASSES=0): a pass
computes the same sums in the same order whichever way it is launched, but the one- and two-pass kernels are separate
instantiations whose epilogues the compiler may contract into fused multiply-adds differently, so the two runs agree
to a few units in the last place of fp32 (asserted: a fifth of the tolerance against the oracle), not bit for bit."""
import numpy as np
import pytest

import easyspec_synth as synth
from tolerances import TOL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device; none is visible")
    import gpu_harness
    return gpu_harness


def run_case(oracle, gpu, monkeypatch, cfg, seed, ctxs, n_calib, max_calib, pairs, fuzzy_first=1):
    """Sequences with KV prefixes of ctxs slots take fuzzy_first fuzzy steps, then sequence b is calibrated with
    n_calib[b] tokens (0 = left alone), once with paired passes and once one pass at a time.  pairs: how many pairs of
    passes the calibration must form, checked by counting its launches: a pair saves the QKV, O, gate/up and down
    launches of every layer and the head launch of one pass."""
    import paper_2502_02493_amd as es
    B = len(ctxs)
    w = synth.make_weights(cfg, seed)
    max_ctx = max(ctxs) + fuzzy_first + max_calib + 8
    model = oracle.Model(cfg, w, max_ctx)
    toks = synth.make_tokens(seed + 1, B * (max_calib + fuzzy_first), cfg["vocab"]).reshape(B, -1)
    bounds = np.array([0, 1, cfg["n_layers"] - 1, cfg["n_layers"]], np.int32)
    results = []
    for pair in ("1", "0"):
        monkeypatch.setenv("EASYSPEC_PAIR_PASSES", pair)
        g = gpu.GpuDrafter(cfg, w, max_batch=B, max_ctx=max_ctx, max_calib=max_calib)
        try:
            g.set_groups(bounds)
            for b, n in enumerate(ctxs):
                k, v = synth.make_kv_prefix(cfg, seed + 2, n, seq=b)
                g.import_kv(b, k, v)
            for step in range(fuzzy_first):
                g.draft_step({b: int(toks[b, step]) for b in range(B)})
            calib = {b: [int(t) for t in toks[b, fuzzy_first:fuzzy_first + n]] for b, n in enumerate(n_calib) if n > 0}
            es.easyspec_profile_begin(g.ctx, es.EASYSPEC_OP_ALL, 8192)
            gt, gl = g.calibrate(calib, all_rows=True)
            launches = es.easyspec_profile_end(g.ctx)[0]
            kv = {b: g.export_kv(b, ctxs[b] + n_calib[b]) for b in calib}
            results.append((gt, gl, kv, g.lens(), launches))
        finally:
            g.close()
    (gt1, gl1, kv1, lens1, launches1), (gt0, gl0, kv0, lens0, launches0) = results
    assert launches0 - launches1 == pairs * (4 * cfg["n_layers"] + 1), (launches0, launches1)
    tol = TOL[cfg["dtype"]]
    kv_tol = max(tol, 2e-3) if cfg["dtype"] == "bf16" else tol   # a bf16 entry may differ by one unit in the last place
    for b in gl1:
        gpu.assert_close(gl1[b], gl0[b], tol / 5, f"sequence {b}: paired against single passes")
        for x1, x0 in zip(kv1[b], kv0[b]):
            assert gpu.rel_l2(x1, x0) < kv_tol / 5
    assert np.array_equal(lens1[0], lens0[0]) and np.array_equal(lens1[1], lens0[1])
    # against the oracle, one sequence at a time
    for b, n in enumerate(n_calib):
        so = oracle.Sequence(model)
        k, v = synth.make_kv_prefix(cfg, seed + 2, ctxs[b], seq=b)
        so.import_kv(k, v)
        for step in range(fuzzy_first):
            so.fuzzy_step(bounds, int(toks[b, step]))
        if n == 0:
            assert (int(lens1[0][b]), int(lens1[1][b])) == (so.precise, so.fuzzy)
            continue
        wl = so.calibrate([int(t) for t in toks[b, fuzzy_first:fuzzy_first + n]], all_rows=True)
        gpu.assert_close(gl1[b], wl, tol, f"calibration logits, sequence {b}")
        assert (int(lens1[0][b]), int(lens1[1][b])) == (so.precise, 0)
        kk, vv = kv1[b]
        assert gpu.rel_l2(kk, so.K[:, :, :so.precise]) < kv_tol
        assert gpu.rel_l2(vv, so.V[:, :, :so.precise]) < kv_tol


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_four_sequences_of_six_tokens(oracle, gpu, monkeypatch, dtype):
    """The long-context batch's calibration in small: 4 x 6 tokens = two passes of 12 columns (two fragments each), run as a pair."""
    run_case(oracle, gpu, monkeypatch, synth.model_shape("tiny", dtype=dtype), 1100, [40, 300, 7, 129], [6, 6, 6, 6], 6, pairs=1)


def test_odd_number_of_passes_and_an_idle_sequence(oracle, gpu, monkeypatch):
    """5 x 8 tokens with one sequence left alone: passes of 16, 16 and 8 columns, the first two as a pair, the third alone."""
    run_case(oracle, gpu, monkeypatch, synth.model_shape("tiny", dtype="bf16"), 1110, [33, 64, 5, 257, 90, 12], [8, 8, 0, 8, 8, 8], 8, pairs=1)


def test_unequal_passes_run_one_at_a_time(oracle, gpu, monkeypatch):
    """Passes of 15, 9 + 5 = 14 and 16 columns: no two consecutive passes are equal, none is paired."""
    run_case(oracle, gpu, monkeypatch, synth.model_shape("tiny", dtype="bf16"), 1120, [20, 270, 66, 31], [15, 9, 5, 16], 16, pairs=0)


def test_pairs_of_folded_passes_qwen_shape(oracle, gpu, monkeypatch):
    """Eight sequences of 4 tokens on the Qwen-like shape (QKV bias, 7 heads per KV head): passes of 16 + 16, one pair;
    then 6 sequences of 3 tokens with max_calib 3: 15 + 3 columns, unequal."""
    cfg = synth.model_shape("tiny_qwen", dtype="bf16")
    run_case(oracle, gpu, monkeypatch, cfg, 1130, [9, 100, 258, 31, 64, 300, 2, 77], [4] * 8, 4, pairs=1)
    run_case(oracle, gpu, monkeypatch, cfg, 1131, [9, 100, 258, 31, 64, 300], [3] * 6, 3, pairs=0)


def test_sixteen_and_eight_columns(oracle, gpu, monkeypatch):
    """6 x 4 tokens fill a pass of 16 columns and one of 8 (whose lo terms fold into the same MFMA: another launch
    shape), so nothing is paired.  (Two consecutive passes of at most 8 columns each cannot occur: they would have
    been one pass.)"""
    run_case(oracle, gpu, monkeypatch, synth.model_shape("tiny", dtype="bf16"), 1140, [50, 260, 17, 140, 8, 99], [4] * 6, 4, pairs=0, fuzzy_first=2)


def test_8b_layer_shape_reduced_depth(oracle, gpu, monkeypatch):
    """The 8B layer shape (real tile counts, wave counts and seven-wave down projection) at 3 layers: 4 x 6 tokens."""
    cfg = synth.model_shape("llama3_8b", n_layers=3, vocab=4096)
    run_case(oracle, gpu, monkeypatch, cfg, 1150, [300, 40, 700, 129], [6, 6, 6, 6], 6, pairs=1)


def test_four_passes_two_pairs(oracle, gpu, monkeypatch):
    """8 x 8 tokens: four passes of 16 columns, run as two pairs one after the other (the second pair reuses both
    workspace sets)."""
    run_case(oracle, gpu, monkeypatch, synth.model_shape("tiny", dtype="bf16"), 1160, [12, 70, 257, 3, 129, 64, 300, 31], [8] * 8, 8, pairs=2)
